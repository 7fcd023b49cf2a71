/*
 * seka.h — C ABI of the MI355X (gfx950) SEKA / AdaSEKA prefill library.
 *
 * The library computes causal grouped-query prefill attention whose keys are spectrally
 * edited before scoring (paper Sec. 2: k'_j = k_j + g P k_j on highlighted tokens j, one
 * projector P per (layer, KV head); Sec. 3.3: for AdaSEKA P = sum_m alpha_m U_m U_m^T).
 *
 * General conventions (all entry points):
 *   - Tensors are row-major [B, S, H, D] (batch, token, head, head dim; the layout of the
 *     key-editing hook's input in Algorithms 1 and 2), D contiguous.  Query head hq reads
 *     KV head hq / (Hq / Hkv).
 *   - "dev" pointers are device (HBM) addresses on the current HIP device, owned by the caller,
 *     16-byte aligned.  "host" pointers are ordinary host memory, read before the call returns.
 *   - Calls validate their arguments on the host first (no GPU work is issued on error), then
 *     enqueue kernels on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and return without waiting.  The library never allocates or frees device memory.
 *   - Inputs are never written.  Outputs must not overlap inputs unless stated.
 *   - Size limits beyond those stated per call (SEKA_ERR_SHAPE): S * H * D < 2^31 elements per prompt;
 *     B * Hkv <= 65535 for the routing calls, B <= 65535 for the edit and decode calls, B * S / 128 <= 65535
 *     for seka_project_route (their launch grids carry these on an axis that HIP limits to 65535).
 *   - Return value: SEKA_OK or an error code; seka_status_string() names it.
 */
#ifndef SEKA_H
#define SEKA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SEKA_OK = 0,
  SEKA_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  SEKA_ERR_SHAPE = 2,       /* a dimension is out of range or inconsistent                 */
  SEKA_ERR_DTYPE = 3,       /* unknown element type                                        */
  SEKA_ERR_ALIGN = 4,       /* a device pointer is not 16-byte aligned                     */
  SEKA_ERR_ALIAS = 5,       /* an output overlaps an input in a way that is not allowed    */
  SEKA_ERR_UNSUPPORTED = 6, /* valid request that this build has no kernel for             */
  SEKA_ERR_LAUNCH = 7,      /* the HIP runtime reported an error on launch                 */
  SEKA_ERR_WORKSPACE = 8    /* workspace missing or too small                              */
} seka_status;

typedef enum { SEKA_F32 = 0, SEKA_BF16 = 1 } seka_dtype;

typedef enum {
  SEKA_ROUTE_SOFTMAX_COS = 0, /* w = softmax_m(tau * cos(q_bar, prototype_m))                */
  SEKA_ROUTE_PAPER_EQ6 = 1    /* alpha_m = <q_bar, p_m> / max_m' |<q_bar, p_m'>|  (Eq. 6)    */
} seka_route_mode;

enum { SEKA_MAX_RANK = 128, SEKA_MAX_KV_HEADS = 64, SEKA_MAX_EXPERTS = 16 };

/* Problem shape.  D must be 64 or 128; Hq must be a multiple of Hkv; Hkv <= SEKA_MAX_KV_HEADS. */
typedef struct {
  int32_t B, S, Hq, Hkv, D;
  int32_t dtype;          /* seka_dtype: element type of Q, K, V, O and U                      */
  float softmax_scale;    /* scores are scale * q.k; <= 0 selects 1/sqrt(D) (paper Sec. 2)     */
} seka_shape;

/* Steering of one layer (paper Algorithm 1 hook inputs; Algorithm 2 for M > 1). */
typedef struct {
  int32_t M;              /* experts per KV head; 1 = SEKA                                     */
  int32_t r;              /* retained columns per expert; M*r <= SEKA_MAX_RANK; for bf16 tensors
                             r must be a multiple of 8 (pad U with zero columns otherwise)     */
  const void* U;          /* dev [Hkv, M, D, r], tensor dtype: column c of U[h,m] is the c-th
                             basis vector of expert m's subspace (Eq. 2: P = U U^T)            */
  const float* w;         /* dev [B, Hkv, M] fp32 routing coefficients (output of seka_route),
                             or NULL for all ones (SEKA)                                       */
  const float* gain;      /* host [Hkv] fp32: g of k' = k + g P k; any real value; 0 means the
                             head is not selected for steering (paper Sec. 3.4)                */
  const uint8_t* mask;    /* dev [B, S]: nonzero = highlighted token (Algorithm 1, "if m_{b,t}
                             = 1"); shared by all heads                                        */
  const float* key_scale; /* host [Hkv] fp32 or NULL for all ones: a of k' = a k + g P k on
                             highlighted tokens of steered heads (gain != 0).  Eq. 4 with a
                             negative-side gain is this form: its projector onto the trailing
                             singular vectors is I minus the projector onto the leading ones,
                             so k' = (1 + g-/2) k + (g+/2) P+ k - (g-/2) P-lead k: two experts
                             with coefficients w = (g+/2, -g-/2), gain 1, key_scale 1 + g-/2  */
} seka_steer;

/*
 * seka_route — AdaSEKA expert coefficients from the prompt's queries (paper Sec. 3.3, Eq. 6).
 *
 * q_bar[b,h,:] = mean of Q[b, t, hq, :] over tokens t in [t0, t1) and over the Hq/Hkv query
 * heads hq of KV head h.  Then per (b, h):
 *   SOFTMAX_COS: w_m = softmax_m(tau * <q_bar, p_m> / (|q_bar| |p_m|)); a product of norms
 *                below 1e-30 gives cos = 0.
 *   PAPER_EQ6:   alpha_m = <q_bar, p_m> / max_m' |<q_bar, p_m'>| with p_m = sum_k sigma_m^(k)
 *                u_m^(k) precomputed by the caller (the K-term sum of Eq. 6 is linear in q);
 *                all-zero alignments (max < 1e-30) give alpha = 0.  The paper uses the last
 *                prompt token: [t0, t1) = [S-1, S).  tau is ignored.
 *
 * Q      dev [B,S,Hq,D] tensor dtype.          proto  dev [Hkv,M,D] fp32.
 * w_out  dev [B,Hkv,M] fp32 (written).         1 <= M <= SEKA_MAX_EXPERTS, 0 <= t0 < t1 <= S.
 * workspace  dev scratch of at least seka_route_workspace_bytes(sh, t0, t1) bytes, 16-byte
 *            aligned; contents on return are unspecified.  Calls sharing a workspace must be
 *            ordered by their stream.
 */
size_t seka_route_workspace_bytes(const seka_shape* sh, int32_t t0, int32_t t1);
seka_status seka_route(const void* Q, const seka_shape* sh, const float* proto, int32_t M,
                       int32_t t0, int32_t t1, int32_t mode, float tau, float* w_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * seka_route_ragged — seka_route for a batch whose prompts differ in length (paper Sec. 3.3: the query that
 * routes is taken at the end of each prompt, so its position differs per prompt).  For prompt b the mean runs
 * over its last `window` tokens, t in [max(0, len_b - window), len_b): window = 1 is the paper's last prompt
 * token, window >= S the whole prompt.  Everything else is seka_route.
 *
 * cu_seqlens == NULL: Q dev [B,S,Hq,D] (padded); len_b = seq_lens[b], seq_lens dev [B] int32 (required).
 * cu_seqlens != NULL: Q dev [total_tokens,Hq,D] (packed); cu_seqlens dev [B+1] int32, ascending, cu[0] = 0,
 *                     cu[B] = total_tokens; prompt b is rows cu[b] .. cu[b+1]-1; seq_lens is ignored and
 *                     sh->S is the longest prompt.  Rows are clamped to the tensor on the device.
 * len_b is clamped to [0, S].  A prompt without tokens has q_bar = 0: SOFTMAX_COS gives 1/M for every expert,
 * PAPER_EQ6 gives 0.
 * workspace  dev scratch of at least seka_route_ragged_workspace_bytes(sh, window) bytes, 16-byte aligned.
 * Errors as seka_route; both length arrays NULL is SEKA_ERR_NULL, window < 1 SEKA_ERR_SHAPE.
 */
size_t seka_route_ragged_workspace_bytes(const seka_shape* sh, int32_t window);
seka_status seka_route_ragged(const void* Q, const seka_shape* sh, const float* proto, int32_t M,
                              const int32_t* seq_lens, const int32_t* cu_seqlens, int64_t total_tokens,
                              int32_t window, int32_t mode, float tau, float* w_out, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * seka_project_route — the query projection with AdaSEKA's routing in its epilogue (paper Sec. 3.3: the
 * routing query is formed from the layer's queries, which this projection has just produced, so the separate
 * pass of seka_route over Q is not needed).
 *   Q_out[b,t,hq,d] = sum_e X[b,t,e] Wq[hq*D + d, e]      (fp32 accumulation, rounded once to bf16)
 *   w_out = seka_route(Q_out, t0 = 0, t1 = S, mode, tau)    (from the rounded values, without reading them back)
 *
 * X      dev [B,S,E] bf16: the layer's input tokens.     Wq  dev [Hq*D, E] bf16: one row per output feature.
 * Q_out  dev [B,S,Hq,D] bf16 (written).                  E: a multiple of 64.
 * w_out  dev [B,Hkv,M] fp32 or NULL (projection only; proto, M, mode, tau and the workspace are then ignored).
 * proto, M, mode, tau as in seka_route.
 * workspace  dev scratch of at least seka_project_route_workspace_bytes(sh) bytes, 16-byte aligned.
 * bf16, D = 128 and S a multiple of 128 only (SEKA_ERR_UNSUPPORTED otherwise; the size call then returns 0).
 */
size_t seka_project_route_workspace_bytes(const seka_shape* sh);
seka_status seka_project_route(const void* X, const void* Wq, int32_t E, void* Q_out, const seka_shape* sh,
                               const float* proto, int32_t M, int32_t mode, float tau, float* w_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * seka_edit_keys — the standalone key-editing hook (Algorithm 1 / 2, inference part):
 *   K_out[b,t,h,:] = K_in[b,t,h,:] + gain[h] * sum_m w[b,h,m] U[h,m] (U[h,m]^T K_in[b,t,h,:])
 * where mask[b,t] != 0 and gain[h] != 0; K_out = K_in elsewhere.
 *
 * K_in, K_out  dev [B,S,Hkv,D] tensor dtype.  K_out == K_in is allowed (then only highlighted
 * rows of selected heads are written); any other overlap returns SEKA_ERR_ALIAS.
 * sh->Hq is ignored.  Accumulation is fp32; the result is rounded once to the tensor dtype.
 */
seka_status seka_edit_keys(const void* K_in, void* K_out, const seka_shape* sh,
                           const seka_steer* st, void* hip_stream);

/*
 * seka_edit_keys_packed — seka_edit_keys for prompts stored back to back (the layout of
 * seka_attention_prefill_packed), so that the edited keys of an unpadded batch can persist in its cache with
 * per-prompt expert weights (paper Sec. 3.3: the routing coefficients differ per prompt).
 *
 * K_in, K_out  dev [total_tokens,Hkv,D]; K_out == K_in allowed, any other overlap is SEKA_ERR_ALIAS.
 * cu_seqlens   dev [B+1] int32, ascending, cu[0] = 0, cu[B] <= total_tokens: prompt b is rows cu[b] .. cu[b+1]-1.
 *              Offsets are clamped into the tensor on the device; rows that belong to no prompt, and rows of a
 *              prompt beyond sh->S (the longest prompt the launch covers), are not touched.
 * st->mask     dev [total_tokens]; st->w dev [B,Hkv,M] (indexed by prompt).  Everything else as seka_edit_keys.
 */
seka_status seka_edit_keys_packed(const void* K_in, void* K_out, const seka_shape* sh, const seka_steer* st,
                                  const int32_t* cu_seqlens, int64_t total_tokens, void* hip_stream);

/*
 * seka_attention_prefill — causal attention on the edited keys, edit fused in (paper Sec. 2 and
 * Eq. 5: logits_ij = q_i . k'_j / sqrt(d_k), j <= i; softmax over j; O_i = sum_j p_ij v_j).
 * K itself is not modified: edited keys exist only on chip, or not at all: for bf16, D = 128,
 * M * r <= 32 and unit key scales the same logits are formed on the score side,
 * q_i . k_j + (U^T q_i) . (c .* U^T k_j) for highlighted j (the equivalence stated in Sec. 2).
 *
 * Q, O  dev [B,S,Hq,D];  K, V  dev [B,S,Hkv,D];  all tensor dtype.
 * lse   dev [B,Hq,S] fp32 or NULL: natural log of the softmax denominator (row maximum included).
 * st == NULL, st->mask == NULL or all gains zero gives exactly seka_attention_plain.
 * bf16 tensors: products on the matrix cores with fp32 accumulation, softmax in fp32.
 */
seka_status seka_attention_prefill(const void* Q, const void* K, const void* V, void* O,
                                   float* lse, const seka_shape* sh, const seka_steer* st,
                                   void* hip_stream);

/* seka_attention_plain — the same attention with unedited keys (the unsteered baseline). */
seka_status seka_attention_plain(const void* Q, const void* K, const void* V, void* O, float* lse,
                                 const seka_shape* sh, void* hip_stream);

/*
 * seka_attention_prefill_ragged — seka_attention_prefill for a padded batch of prompts of different lengths:
 * prompt b has seq_lens[b] tokens (clamped to [0, S]); tokens at and beyond that index are padding: they are
 * neither queries nor keys, and their rows of O and lse are left untouched.  The tensors keep their [B,S,...]
 * layout (S = padded length).  seq_lens dev [B] int32, or NULL for seka_attention_prefill; st may be NULL for
 * unsteered attention.
 */
seka_status seka_attention_prefill_ragged(const void* Q, const void* K, const void* V, void* O, float* lse,
                                          const seka_shape* sh, const seka_steer* st, const int32_t* seq_lens,
                                          void* hip_stream);

/*
 * seka_attention_prefill_packed — seka_attention_prefill for a batch stored without padding (the "varlen"
 * layout of serving stacks): the prompts' tokens follow one another in tensors of total_tokens rows, prompt b
 * owning rows [cu_seqlens[b], cu_seqlens[b+1]).
 *
 * Q, O      dev [total_tokens,Hq,D];  K, V dev [total_tokens,Hkv,D];  st->mask dev [total_tokens];
 * lse       dev [Hq,total_tokens] fp32 or NULL;  st->w stays [B,Hkv,M] (one set of coefficients per prompt).
 * sh->B     number of prompts; sh->S an upper bound of the longest prompt (it sizes the launch; longer prompts
 *           are cut to sh->S tokens).
 * cu_seqlens dev [B+1] int32, non-decreasing, cu_seqlens[0] = 0 expected; values are clamped into
 *           [0, total_tokens] on the device, so no content of it can make the kernels leave the tensors.
 * st may be NULL for unsteered attention.  Rows of O / lse that belong to no prompt are left untouched.
 * (seka_edit_keys serves this layout as B = 1, S = total_tokens when w is NULL; seka_route per prompt.)
 */
seka_status seka_attention_prefill_packed(const void* Q, const void* K, const void* V, void* O, float* lse,
                                          const seka_shape* sh, const seka_steer* st, const int32_t* cu_seqlens,
                                          int64_t total_tokens, void* hip_stream);

/*
 * seka_attention_decode — the generation step after a steered prefill.  The edited keys persist in the KV
 * cache (run seka_edit_keys in place on the prompt's keys, the hook of Algorithm 1), so the new token's query
 * attends to the cache as it is: logits q . k_j / sqrt(d_k) over the first seq_lens[b] cached tokens (its own
 * key included), softmax, O = sum_j p_j v_j (paper Sec. 2).  Memory-bound: K and V are read once.
 *
 * q, O      dev [B,Hq,D] tensor dtype (one query per prompt and head).
 * K, V      dev [B,S,Hkv,D] tensor dtype: the caches; sh->S is their capacity in tokens.
 * lse       dev [B,Hq] fp32 or NULL.
 * seq_lens  dev [B] int32 or NULL (= S for every prompt); values are clamped to [0, S]; a prompt with no
 *           cached token gets O = 0 and lse = -inf.
 * workspace dev scratch of at least seka_decode_workspace_bytes(sh) bytes, 16-byte aligned; contents on return
 *           are unspecified; calls sharing it must be ordered by their stream.  (Caches short enough to be
 *           taken in one piece per head group, S < 1024, are one kernel that does not touch it.)
 */
size_t seka_decode_workspace_bytes(const seka_shape* sh);
seka_status seka_attention_decode(const void* q, const void* K, const void* V, void* O, float* lse,
                                  const int32_t* seq_lens, const seka_shape* sh, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

/*
 * seka_attention_decode_static — seka_attention_decode for callers that cannot allocate device memory or size a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors, without the workspace pair: the partial states go to a buffer of
 * SEKA_DECODE_STATIC_MAX_BYTES (8 MiB) that the library owns in device memory (one per GPU that loads the
 * library, held until the process ends).  The call allocates and frees nothing.
 *   - Problems whose partial states exceed the buffer (seka_decode_workspace_bytes(sh) > SEKA_DECODE_STATIC_MAX_BYTES;
 *     B * Hq * splits * (D + 2) * 4 bytes with at most 64 splits, e.g. more than 256 (prompt, query head) pairs
 *     of a long cache at D = 128) return SEKA_ERR_WORKSPACE and launch nothing: use seka_attention_decode.
 *   - Every call on a GPU shares that GPU's buffer.  Calls on one stream are ordered by it; calls that overlap
 *     in time on one GPU (different streams, no dependency) race on the buffer and give wrong results.  Nothing
 *     in the buffer has to start at zero: every slot a launch reads is written earlier in the same call.
 *   - The first call on a device looks the buffer's address up (no allocation); make it before a capture begins.
 */
enum { SEKA_DECODE_STATIC_MAX_BYTES = 8 << 20 };
seka_status seka_attention_decode_static(const void* q, const void* K, const void* V, void* O, float* lse,
                                         const int32_t* seq_lens, const seka_shape* sh, void* hip_stream);

/*
 * seka_learn_projection — the offline stage for one layer (paper Sec. 3.1): per KV head, the cross-covariance
 * Omega_h = h_neutral^T h_signal / n of token key embeddings sampled under a neutral and under a relevant
 * (or irrelevant) context, its singular value decomposition Omega = U Sigma V^T, and the rank k_h that keeps a
 * share gamma of the singular-value mass (Eq. 3: the smallest k with sum_{i<=k} sigma_i >= gamma sum_i sigma_i).
 * The positive projector of Eq. 2 is P = U[:, :k] U[:, :k]^T; for the negative projector pass the irrelevant
 * samples as h_signal and keep the trailing columns U[:, k:].
 *
 * h_neutral, h_signal  dev [B,S,Hkv,D] tensor dtype: n = B*S paired sample tokens (row t of both is the same
 *                      token under the two contexts); n < 2^24.
 * gamma      in (0, 1].
 * U_out      dev [Hkv,D,D] fp32: column c of U_out[h] is the left singular vector of the c-th largest singular
 *            value (unit norm, sign unspecified).  Where sigma_c <= 1e-5 sigma_1 no direction is determined in
 *            fp32 and the column is all zero; vectors of equal singular values span the right subspace only.
 * sigma_out  dev [Hkv,D] fp32, descending.
 * k_out      dev [Hkv] int32, in [1, D].
 * U_packed   dev [Hkv,D,r_pad] tensor dtype or NULL: the first min(k_h, r_pad) columns of U_out[h], the remaining
 *            columns zero, ready to be seka_steer.U with M = 1, r = r_pad (1 <= r_pad <= D).
 * workspace  dev scratch of at least seka_learn_workspace_bytes(sh) bytes, 16-byte aligned.
 * fp32 arithmetic throughout (one-sided Jacobi iteration to a relative off-diagonal of 2e-6); deterministic.
 * The decomposition runs one workgroup per head and is bound by its own latency, so a call costs about the
 * same for 8 heads as for 64: heads of several layers may be stacked along the head axis of one call (Hkv <=
 * SEKA_MAX_KV_HEADS).
 *
 * seka_head_distance — the head-selection score of Sec. 3.4: D_out[h] = (1/n) sum_t || h_pos[t,h,:] -
 * h_neg[t,h,:] ||_2 over the n = B*S sample tokens; heads whose score clears a threshold are given a nonzero
 * gain by the caller.  h_pos, h_neg dev [B,S,Hkv,D] tensor dtype; D_out dev [Hkv] fp32; workspace as above
 * (seka_learn_workspace_bytes covers both calls).  Deterministic.
 */
size_t seka_learn_workspace_bytes(const seka_shape* sh);
seka_status seka_learn_projection(const void* h_neutral, const void* h_signal, const seka_shape* sh, float gamma,
                                  float* U_out, float* sigma_out, int32_t* k_out, void* U_packed, int32_t r_pad,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);
seka_status seka_head_distance(const void* h_pos, const void* h_neg, const seka_shape* sh, float* D_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Name of a status code; static storage, never NULL. */
const char* seka_status_string(int32_t status);

/* HIP runtime's description of the calling thread's most recent launch result ("no error" after a
 * success); for diagnosing SEKA_ERR_LAUNCH.  Static storage, never NULL. */
const char* seka_last_launch_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SEKA_H */
