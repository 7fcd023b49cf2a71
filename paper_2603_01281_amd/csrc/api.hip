// C ABI of libseka: host-side argument validation and dispatch to the HIP launchers.
// Every check here runs before any GPU work is issued, so error paths need no GPU.
#include <cmath>
#include <cstring>

#include "common.h"

namespace {

thread_local hipError_t g_last_hip_error = hipSuccess;

seka_status launch_status(hipError_t e) {
  g_last_hip_error = e;
  if (e == hipSuccess) return SEKA_OK;
  return e == hipErrorNotSupported ? SEKA_ERR_UNSUPPORTED : SEKA_ERR_LAUNCH;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline size_t elem_size(int dtype) { return dtype == SEKA_BF16 ? 2 : 4; }

// Launch grids put the batch (or batch x KV heads) on the y or z axis, which HIP limits to 65535 workgroups.
constexpr int64_t kMaxGridYZ = 65535;

seka_status check_shape(const seka_shape* sh, bool need_q_heads) {
  if (!sh) return SEKA_ERR_NULL;
  if (sh->dtype != SEKA_F32 && sh->dtype != SEKA_BF16) return SEKA_ERR_DTYPE;
  if (sh->B < 1 || sh->S < 1 || sh->Hkv < 1 || sh->Hkv > SEKA_MAX_KV_HEADS) return SEKA_ERR_SHAPE;
  if (sh->D != 64 && sh->D != 128) return SEKA_ERR_SHAPE;
  if (need_q_heads && (sh->Hq < 1 || sh->Hq % sh->Hkv != 0)) return SEKA_ERR_SHAPE;
  if (!std::isfinite(sh->softmax_scale)) return SEKA_ERR_SHAPE;
  // 32-bit element indexing inside one (batch) slice is assumed by the kernels
  const int64_t heads = need_q_heads ? sh->Hq : sh->Hkv;
  if ((int64_t)sh->S * heads * sh->D >= ((int64_t)1 << 31)) return SEKA_ERR_SHAPE;
  return SEKA_OK;
}

seka_status check_steer(const seka_steer* st, const seka_shape* sh) {
  if (!st->U || !st->gain || !st->mask) return SEKA_ERR_NULL;
  if (st->M < 1 || st->M > SEKA_MAX_EXPERTS || st->r < 1) return SEKA_ERR_SHAPE;
  if ((int64_t)st->M * st->r > SEKA_MAX_RANK) return SEKA_ERR_SHAPE;
  if (st->r > sh->D) return SEKA_ERR_SHAPE;
  if (misaligned(st->U) || (st->w && misaligned(st->w))) return SEKA_ERR_ALIGN;
  for (int h = 0; h < sh->Hkv; ++h) {
    if (!std::isfinite(st->gain[h])) return SEKA_ERR_SHAPE;
    if (st->key_scale && !std::isfinite(st->key_scale[h])) return SEKA_ERR_SHAPE;
  }
  if (sh->dtype == SEKA_BF16 && st->r % 8 != 0) return SEKA_ERR_UNSUPPORTED;
  return SEKA_OK;
}

void fill_steer(seka::SteerArgs& sa, const seka_steer* st, int Hkv) {
  std::memset(&sa, 0, sizeof(sa));
  sa.U = st->U;
  sa.w = st->w;
  sa.mask = st->mask;
  sa.M = st->M;
  sa.r = st->r;
  for (int h = 0; h < Hkv; ++h) {
    sa.gain[h] = st->gain[h];
    sa.kscale[h] = st->key_scale ? st->key_scale[h] : 1.0f;
  }
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + nb && y < x + na;
}

// seq_lens: padded batch with per-prompt lengths; cu_seqlens (with total_tokens): packed batch; at most one of them.
seka_status attention_common(const void* Q, const void* K, const void* V, void* O, float* lse,
                             const seka_shape* sh, const seka_steer* st, const int32_t* seq_lens,
                             const int32_t* cu_seqlens, int64_t total_tokens, void* hip_stream) {
  seka_status rc = check_shape(sh, true);
  if (rc != SEKA_OK) return rc;
  if (!Q || !K || !V || !O) return SEKA_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || (lse && misaligned(lse)))
    return SEKA_ERR_ALIGN;
  if (seq_lens && (reinterpret_cast<uintptr_t>(seq_lens) & 3u)) return SEKA_ERR_ALIGN;
  if (cu_seqlens && (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u)) return SEKA_ERR_ALIGN;
  if (cu_seqlens && (total_tokens < 1 || total_tokens > 0x7fffffffLL)) return SEKA_ERR_SHAPE;
  const size_t es = elem_size(sh->dtype);
  const size_t tokens = cu_seqlens ? (size_t)total_tokens : (size_t)sh->B * sh->S;
  const size_t nq = tokens * sh->Hq * sh->D * es;
  const size_t nk = tokens * sh->Hkv * sh->D * es;
  if (ranges_overlap(O, nq, Q, nq) || ranges_overlap(O, nq, K, nk) || ranges_overlap(O, nq, V, nk))
    return SEKA_ERR_ALIAS;

  bool steered = false;
  seka::SteerArgs sa;
  if (st && st->mask) {
    rc = check_steer(st, sh);
    if (rc != SEKA_OK) return rc;
    for (int h = 0; h < sh->Hkv; ++h) steered |= (st->gain[h] != 0.0f);
    if (steered) fill_steer(sa, st, sh->Hkv);
  }

  seka::AttnArgs a;
  a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse; a.lens = seq_lens;
  a.cu = cu_seqlens; a.total = cu_seqlens ? (int)total_tokens : 0;
  a.B = sh->B; a.S = sh->S; a.Hq = sh->Hq; a.Hkv = sh->Hkv; a.D = sh->D;
  a.scale = sh->softmax_scale > 0.0f ? sh->softmax_scale : 1.0f / std::sqrt((float)sh->D);
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  (void)hipGetLastError();   // drop any stale error left by earlier, unrelated runtime calls of this thread
  hipError_t e = (sh->dtype == SEKA_BF16)
                     ? seka::launch_attention_bf16(a, steered ? &sa : nullptr, stream)
                     : seka::launch_attention_f32(a, steered ? &sa : nullptr, stream);
  return launch_status(e);
}

}  // namespace

extern "C" {

const char* seka_status_string(int32_t status) {
  switch (status) {
    case SEKA_OK: return "ok";
    case SEKA_ERR_NULL: return "a required pointer is NULL";
    case SEKA_ERR_SHAPE: return "a dimension or scalar argument is out of range";
    case SEKA_ERR_DTYPE: return "unknown element type";
    case SEKA_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case SEKA_ERR_ALIAS: return "an output overlaps an input";
    case SEKA_ERR_UNSUPPORTED: return "no kernel for this request";
    case SEKA_ERR_LAUNCH: return "HIP reported an error on launch";
    case SEKA_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

const char* seka_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

size_t seka_route_workspace_bytes(const seka_shape* sh, int32_t t0, int32_t t1) {
  if (check_shape(sh, true) != SEKA_OK || t0 < 0 || t1 <= t0 || t1 > sh->S) return 0;
  return seka::route_workspace_bytes(sh->B, sh->Hkv, sh->D, t0, t1);
}

seka_status seka_route(const void* Q, const seka_shape* sh, const float* proto, int32_t M, int32_t t0,
                       int32_t t1, int32_t mode, float tau, float* w_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  seka_status rc = check_shape(sh, true);
  if (rc != SEKA_OK) return rc;
  if (!Q || !proto || !w_out) return SEKA_ERR_NULL;
  if (M < 1 || M > SEKA_MAX_EXPERTS) return SEKA_ERR_SHAPE;
  if (t0 < 0 || t1 <= t0 || t1 > sh->S) return SEKA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->Hkv > kMaxGridYZ) return SEKA_ERR_SHAPE;
  if (mode != SEKA_ROUTE_SOFTMAX_COS && mode != SEKA_ROUTE_PAPER_EQ6) return SEKA_ERR_UNSUPPORTED;
  if (!std::isfinite(tau)) return SEKA_ERR_SHAPE;
  if (misaligned(Q) || misaligned(proto) || (reinterpret_cast<uintptr_t>(w_out) & 3u)) return SEKA_ERR_ALIGN;
  const size_t need = seka::route_workspace_bytes(sh->B, sh->Hkv, sh->D, t0, t1);
  if (!workspace || workspace_bytes < need) return SEKA_ERR_WORKSPACE;
  if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  (void)hipGetLastError();
  hipError_t e = seka::launch_route(Q, sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype, proto, M, t0, t1, mode,
                                    tau, w_out, workspace, reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

size_t seka_route_ragged_workspace_bytes(const seka_shape* sh, int32_t window) {
  if (check_shape(sh, true) != SEKA_OK || window < 1) return 0;
  return seka::route_workspace_bytes(sh->B, sh->Hkv, sh->D, 0, window < sh->S ? window : sh->S);
}

seka_status seka_route_ragged(const void* Q, const seka_shape* sh, const float* proto, int32_t M,
                              const int32_t* seq_lens, const int32_t* cu_seqlens, int64_t total_tokens,
                              int32_t window, int32_t mode, float tau, float* w_out, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  seka_status rc = check_shape(sh, true);
  if (rc != SEKA_OK) return rc;
  if (!Q || !proto || !w_out) return SEKA_ERR_NULL;
  if (!seq_lens && !cu_seqlens) return SEKA_ERR_NULL;
  if (M < 1 || M > SEKA_MAX_EXPERTS || window < 1) return SEKA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->Hkv > kMaxGridYZ) return SEKA_ERR_SHAPE;
  if (cu_seqlens && (total_tokens < 1 || total_tokens > 0x7fffffffLL)) return SEKA_ERR_SHAPE;
  if (mode != SEKA_ROUTE_SOFTMAX_COS && mode != SEKA_ROUTE_PAPER_EQ6) return SEKA_ERR_UNSUPPORTED;
  if (!std::isfinite(tau)) return SEKA_ERR_SHAPE;
  if (misaligned(Q) || misaligned(proto) || (reinterpret_cast<uintptr_t>(w_out) & 3u)) return SEKA_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(seq_lens) & 3u) || (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u)) return SEKA_ERR_ALIGN;
  const int win = window < sh->S ? window : sh->S;
  const size_t need = seka::route_workspace_bytes(sh->B, sh->Hkv, sh->D, 0, win);
  if (!workspace || workspace_bytes < need) return SEKA_ERR_WORKSPACE;
  if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  (void)hipGetLastError();
  hipError_t e = seka::launch_route(Q, sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype, proto, M, 0, win, mode, tau,
                                    w_out, workspace, reinterpret_cast<hipStream_t>(hip_stream),
                                    cu_seqlens ? nullptr : seq_lens, cu_seqlens, cu_seqlens ? (int)total_tokens : 0, win);
  return launch_status(e);
}

size_t seka_project_route_workspace_bytes(const seka_shape* sh) {
  if (check_shape(sh, true) != SEKA_OK || sh->D != 128 || sh->S % 128 != 0) return 0;
  return seka::project_route_workspace_bytes(sh->B, sh->S, sh->Hq);
}

seka_status seka_project_route(const void* X, const void* Wq, int32_t E, void* Q_out, const seka_shape* sh,
                               const float* proto, int32_t M, int32_t mode, float tau, float* w_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  seka_status rc = check_shape(sh, true);
  if (rc != SEKA_OK) return rc;
  if (!X || !Wq || !Q_out) return SEKA_ERR_NULL;
  if (E < 64 || E % 64 != 0) return SEKA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->S / 128 > kMaxGridYZ || (int64_t)sh->B * sh->Hkv > kMaxGridYZ) return SEKA_ERR_SHAPE;
  if (sh->dtype != SEKA_BF16 || sh->D != 128 || sh->S % 128 != 0) return SEKA_ERR_UNSUPPORTED;
  if ((int64_t)sh->Hq * sh->D * (int64_t)E >= ((int64_t)1 << 40)) return SEKA_ERR_SHAPE;
  if (misaligned(X) || misaligned(Wq) || misaligned(Q_out)) return SEKA_ERR_ALIGN;
  const size_t nx = (size_t)sh->B * sh->S * E * 2, nw = (size_t)sh->Hq * sh->D * E * 2;
  const size_t nq = (size_t)sh->B * sh->S * sh->Hq * sh->D * 2;
  if (ranges_overlap(Q_out, nq, X, nx) || ranges_overlap(Q_out, nq, Wq, nw)) return SEKA_ERR_ALIAS;
  if (w_out) {
    if (!proto) return SEKA_ERR_NULL;
    if (M < 1 || M > SEKA_MAX_EXPERTS) return SEKA_ERR_SHAPE;
    if (mode != SEKA_ROUTE_SOFTMAX_COS && mode != SEKA_ROUTE_PAPER_EQ6) return SEKA_ERR_UNSUPPORTED;
    if (!std::isfinite(tau)) return SEKA_ERR_SHAPE;
    if (misaligned(proto) || (reinterpret_cast<uintptr_t>(w_out) & 3u)) return SEKA_ERR_ALIGN;
    const size_t need = seka::project_route_workspace_bytes(sh->B, sh->S, sh->Hq);
    if (!workspace || workspace_bytes < need) return SEKA_ERR_WORKSPACE;
    if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  }
  (void)hipGetLastError();
  hipError_t e = seka::launch_project_route(X, Wq, E, Q_out, sh->B, sh->S, sh->Hq, sh->Hkv, proto, M, mode, tau, w_out,
                                            workspace, reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

seka_status seka_edit_keys(const void* K_in, void* K_out, const seka_shape* sh, const seka_steer* st,
                           void* hip_stream) {
  seka_status rc = check_shape(sh, false);
  if (rc != SEKA_OK) return rc;
  if (!K_in || !K_out || !st) return SEKA_ERR_NULL;
  if (sh->B > kMaxGridYZ) return SEKA_ERR_SHAPE;
  rc = check_steer(st, sh);
  if (rc != SEKA_OK) return rc;
  if (misaligned(K_in) || misaligned(K_out)) return SEKA_ERR_ALIGN;
  const size_t nk = (size_t)sh->B * sh->S * sh->Hkv * sh->D * elem_size(sh->dtype);
  if (K_in != K_out && ranges_overlap(K_in, nk, K_out, nk)) return SEKA_ERR_ALIAS;
  seka::SteerArgs sa;
  fill_steer(sa, st, sh->Hkv);
  (void)hipGetLastError();
  hipError_t e = seka::launch_edit_keys(K_in, K_out, sh->B, sh->S, sh->Hkv, sh->D, sh->dtype, sa,
                                        reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

seka_status seka_edit_keys_packed(const void* K_in, void* K_out, const seka_shape* sh, const seka_steer* st,
                                  const int32_t* cu_seqlens, int64_t total_tokens, void* hip_stream) {
  seka_status rc = check_shape(sh, false);
  if (rc != SEKA_OK) return rc;
  if (!K_in || !K_out || !st || !cu_seqlens) return SEKA_ERR_NULL;
  if (sh->B > kMaxGridYZ) return SEKA_ERR_SHAPE;
  rc = check_steer(st, sh);
  if (rc != SEKA_OK) return rc;
  if (total_tokens < 1 || total_tokens > 0x7fffffffLL) return SEKA_ERR_SHAPE;
  if (misaligned(K_in) || misaligned(K_out) || (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u)) return SEKA_ERR_ALIGN;
  const size_t nk = (size_t)total_tokens * sh->Hkv * sh->D * elem_size(sh->dtype);
  if (K_in != K_out && ranges_overlap(K_in, nk, K_out, nk)) return SEKA_ERR_ALIAS;
  seka::SteerArgs sa;
  fill_steer(sa, st, sh->Hkv);
  (void)hipGetLastError();
  hipError_t e = seka::launch_edit_keys(K_in, K_out, sh->B, sh->S, sh->Hkv, sh->D, sh->dtype, sa,
                                        reinterpret_cast<hipStream_t>(hip_stream), cu_seqlens, (int)total_tokens);
  return launch_status(e);
}

size_t seka_decode_workspace_bytes(const seka_shape* sh) {
  if (check_shape(sh, true) != SEKA_OK) return 0;
  return seka::decode_workspace_bytes(sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype);
}

namespace {
// Validation shared by the two generation-step entry points; *need = bytes of partial states the launch writes.
seka_status check_decode(const void* q, const void* K, const void* V, void* O, float* lse, const int32_t* seq_lens,
                         const seka_shape* sh, size_t* need) {
  seka_status rc = check_shape(sh, true);
  if (rc != SEKA_OK) return rc;
  if (!q || !K || !V || !O) return SEKA_ERR_NULL;
  if (sh->B > kMaxGridYZ) return SEKA_ERR_SHAPE;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(O)) return SEKA_ERR_ALIGN;
  if ((lse && (reinterpret_cast<uintptr_t>(lse) & 3u)) || (seq_lens && (reinterpret_cast<uintptr_t>(seq_lens) & 3u)))
    return SEKA_ERR_ALIGN;
  const size_t es = elem_size(sh->dtype);
  const size_t nq = (size_t)sh->B * sh->Hq * sh->D * es;
  const size_t nk = (size_t)sh->B * sh->S * sh->Hkv * sh->D * es;
  if (ranges_overlap(O, nq, q, nq) || ranges_overlap(O, nq, K, nk) || ranges_overlap(O, nq, V, nk)) return SEKA_ERR_ALIAS;
  *need = seka::decode_workspace_bytes(sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype);
  return SEKA_OK;
}
}  // namespace

seka_status seka_attention_decode(const void* q, const void* K, const void* V, void* O, float* lse,
                                  const int32_t* seq_lens, const seka_shape* sh, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  size_t need = 0;
  seka_status rc = check_decode(q, K, V, O, lse, seq_lens, sh, &need);
  if (rc != SEKA_OK) return rc;
  if (!workspace || workspace_bytes < need) return SEKA_ERR_WORKSPACE;
  if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  const float scale = sh->softmax_scale > 0.0f ? sh->softmax_scale : 1.0f / std::sqrt((float)sh->D);
  (void)hipGetLastError();
  hipError_t e = seka::launch_decode(q, K, V, O, lse, seq_lens, sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype, scale,
                                     workspace, reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

seka_status seka_attention_decode_static(const void* q, const void* K, const void* V, void* O, float* lse,
                                         const int32_t* seq_lens, const seka_shape* sh, void* hip_stream) {
  size_t need = 0;
  seka_status rc = check_decode(q, K, V, O, lse, seq_lens, sh, &need);
  if (rc != SEKA_OK) return rc;
  if (need > (size_t)SEKA_DECODE_STATIC_MAX_BYTES) return SEKA_ERR_WORKSPACE;   // larger problems: seka_attention_decode
  void* scratch_ptr = nullptr;
  (void)hipGetLastError();
  hipError_t e = seka::decode_static_scratch(&scratch_ptr);
  if (e != hipSuccess) return launch_status(e);
  const float scale = sh->softmax_scale > 0.0f ? sh->softmax_scale : 1.0f / std::sqrt((float)sh->D);
  e = seka::launch_decode(q, K, V, O, lse, seq_lens, sh->B, sh->S, sh->Hq, sh->Hkv, sh->D, sh->dtype, scale, scratch_ptr,
                          reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

size_t seka_learn_workspace_bytes(const seka_shape* sh) {
  if (check_shape(sh, false) != SEKA_OK || (int64_t)sh->B * sh->S >= (1 << 24)) return 0;
  return seka::learn_workspace_bytes(sh->Hkv, sh->D, sh->B * sh->S);
}

seka_status seka_learn_projection(const void* h_neutral, const void* h_signal, const seka_shape* sh, float gamma,
                                  float* U_out, float* sigma_out, int32_t* k_out, void* U_packed, int32_t r_pad,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  seka_status rc = check_shape(sh, false);
  if (rc != SEKA_OK) return rc;
  if ((int64_t)sh->B * sh->S >= (1 << 24)) return SEKA_ERR_SHAPE;
  if (!h_neutral || !h_signal || !U_out || !sigma_out || !k_out) return SEKA_ERR_NULL;
  if (!(gamma > 0.0f && gamma <= 1.0f)) return SEKA_ERR_SHAPE;
  if (U_packed && (r_pad < 1 || r_pad > sh->D)) return SEKA_ERR_SHAPE;
  if (misaligned(h_neutral) || misaligned(h_signal) || misaligned(U_out) || misaligned(sigma_out) ||
      (U_packed && misaligned(U_packed)) || (reinterpret_cast<uintptr_t>(k_out) & 3u))
    return SEKA_ERR_ALIGN;
  const int n = sh->B * sh->S;
  const size_t nh = (size_t)n * sh->Hkv * sh->D * elem_size(sh->dtype);
  const size_t nu = (size_t)sh->Hkv * sh->D * sh->D * sizeof(float), ns = (size_t)sh->Hkv * sh->D * sizeof(float);
  const void* outs[4] = {U_out, sigma_out, k_out, U_packed};
  const size_t out_bytes[4] = {nu, ns, (size_t)sh->Hkv * sizeof(int32_t),
                               U_packed ? (size_t)sh->Hkv * sh->D * r_pad * elem_size(sh->dtype) : 0};
  for (int i = 0; i < 4; ++i) {
    if (!out_bytes[i]) continue;
    if (ranges_overlap(outs[i], out_bytes[i], h_neutral, nh) || ranges_overlap(outs[i], out_bytes[i], h_signal, nh))
      return SEKA_ERR_ALIAS;
    for (int j = i + 1; j < 4; ++j)
      if (out_bytes[j] && ranges_overlap(outs[i], out_bytes[i], outs[j], out_bytes[j])) return SEKA_ERR_ALIAS;
  }
  const size_t need = seka::learn_workspace_bytes(sh->Hkv, sh->D, n);
  if (!workspace || workspace_bytes < need) return SEKA_ERR_WORKSPACE;
  if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  (void)hipGetLastError();
  hipError_t e = seka::launch_learn(h_neutral, h_signal, n, sh->Hkv, sh->D, sh->dtype, gamma, U_out, sigma_out, k_out,
                                    U_packed, r_pad, workspace, reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

seka_status seka_head_distance(const void* h_pos, const void* h_neg, const seka_shape* sh, float* D_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  seka_status rc = check_shape(sh, false);
  if (rc != SEKA_OK) return rc;
  if ((int64_t)sh->B * sh->S >= (1 << 24)) return SEKA_ERR_SHAPE;
  if (!h_pos || !h_neg || !D_out) return SEKA_ERR_NULL;
  if (misaligned(h_pos) || misaligned(h_neg) || (reinterpret_cast<uintptr_t>(D_out) & 3u)) return SEKA_ERR_ALIGN;
  const int n = sh->B * sh->S;
  const size_t nh = (size_t)n * sh->Hkv * sh->D * elem_size(sh->dtype);
  if (ranges_overlap(D_out, (size_t)sh->Hkv * sizeof(float), h_pos, nh) ||
      ranges_overlap(D_out, (size_t)sh->Hkv * sizeof(float), h_neg, nh))
    return SEKA_ERR_ALIAS;
  if (!workspace || workspace_bytes < seka::learn_workspace_bytes(sh->Hkv, sh->D, n)) return SEKA_ERR_WORKSPACE;
  if (misaligned(workspace)) return SEKA_ERR_ALIGN;
  (void)hipGetLastError();
  hipError_t e = seka::launch_head_distance(h_pos, h_neg, n, sh->Hkv, sh->D, sh->dtype, D_out, workspace,
                                            reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status(e);
}

seka_status seka_attention_prefill(const void* Q, const void* K, const void* V, void* O, float* lse,
                                   const seka_shape* sh, const seka_steer* st, void* hip_stream) {
  return attention_common(Q, K, V, O, lse, sh, st, nullptr, nullptr, 0, hip_stream);
}

seka_status seka_attention_plain(const void* Q, const void* K, const void* V, void* O, float* lse,
                                 const seka_shape* sh, void* hip_stream) {
  return attention_common(Q, K, V, O, lse, sh, nullptr, nullptr, nullptr, 0, hip_stream);
}

seka_status seka_attention_prefill_ragged(const void* Q, const void* K, const void* V, void* O, float* lse,
                                          const seka_shape* sh, const seka_steer* st, const int32_t* seq_lens,
                                          void* hip_stream) {
  return attention_common(Q, K, V, O, lse, sh, st, seq_lens, nullptr, 0, hip_stream);
}

seka_status seka_attention_prefill_packed(const void* Q, const void* K, const void* V, void* O, float* lse,
                                          const seka_shape* sh, const seka_steer* st, const int32_t* cu_seqlens,
                                          int64_t total_tokens, void* hip_stream) {
  if (!cu_seqlens) return SEKA_ERR_NULL;
  return attention_common(Q, K, V, O, lse, sh, st, nullptr, cu_seqlens, total_tokens, hip_stream);
}

}  // extern "C"
