// Host side of the C ABI: argument validation and dispatch.  Nothing here
// touches device memory or synchronises; every entry point either returns an
// error before any launch or enqueues its kernels on the caller's stream.
#include <limits.h>

#include "kvzap_internal.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

constexpr int kMaxH = 16;
constexpr int kMaxD = 512;
constexpr int kMaxM = 640;
constexpr size_t kLdsBytes = 160 * 1024;
// positions are 32-bit in the kernels and a block may step up to a few tiles past the end
// before it clamps: keep that arithmetic away from INT_MAX
constexpr int kMaxT = INT_MAX - (1 << 20);

// shape rules shared by kvzap_score and kvzap_decode_evict
int check_attend_shape(int B, int H, int HQ, int max_rows, int window) {
  if (B <= 0 || H <= 0 || HQ <= 0 || max_rows < 0 || window < 0) return KVZAP_ERR_SHAPE;
  if (HQ % H != 0) return KVZAP_ERR_SHAPE;
  if (HQ / H > 16 || (long long)B * H > 65535) return KVZAP_ERR_UNSUPPORTED;
  return KVZAP_OK;
}

int check_scorer_shape(int Dh, int M, int H) {
  if (Dh <= 0 || M < 0 || H <= 0) return KVZAP_ERR_SHAPE;
  if (H > kMaxH || Dh % 64 != 0) return KVZAP_ERR_UNSUPPORTED;
  if (M > 0) {
    if (M % 128 != 0 || M > kMaxM) return KVZAP_ERR_UNSUPPORTED;
  } else {
    if ((size_t)H * ((size_t)Dh * 2 + 64) > kLdsBytes) return KVZAP_ERR_UNSUPPORTED;
  }
  return KVZAP_OK;
}

size_t mask_workspace(int B, int H, int T) {
  const size_t n = (size_t)B * H * kvzap::mask_chunks(T);
  return kvzap::align_up(n * sizeof(int32_t), 256) + kvzap::align_up(n * sizeof(int64_t), 256);
}

}  // namespace

extern "C" {

const char* kvzap_status_string(int status) {
  switch (status) {
    case KVZAP_OK: return "ok";
    case KVZAP_ERR_NULL: return "a required pointer is NULL";
    case KVZAP_ERR_SHAPE: return "invalid size argument";
    case KVZAP_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case KVZAP_ERR_UNSUPPORTED: return "shape outside the supported set";
    case KVZAP_ERR_CAPACITY: return "output capacity too small";
    case KVZAP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KVZAP_ERR_RUNTIME: return "HIP launch failed";
    case KVZAP_ERR_STATIC_LIMIT:
      return "input larger than the built-in scratch of the allocation-free entry point";
    default: return "unknown status";
  }
}

const char* kvzap_version(void) { return "0.1.0"; }

size_t kvzap_workspace_bytes(int which_call, int B, int T, int Dh, int M, int H) {
  if (B <= 0 || H <= 0) return 0;
  if (T <= 0 && which_call != KVZAP_CALL_ATTEND_DECODE && which_call != KVZAP_CALL_TEACHER_SCORES)
    return 0;
  switch (which_call) {
    case KVZAP_CALL_MASK:
      if ((long long)B * H > 65535) return 0;
      return mask_workspace(B, H, T);
    case KVZAP_CALL_DECODE_EVICT:
      if (check_scorer_shape(Dh, M, H) != KVZAP_OK) return 0;
      return kvzap::decode_workspace_bytes(B, Dh, M, H);
    case KVZAP_CALL_SCORE:
      if (check_scorer_shape(Dh, M, H) != KVZAP_OK) return 0;
      // W1 in fragment order, or the first projection's partial sums of a short prompt
      return M > 0 ? kvzap::score_mlp_workspace_bytes((long long)(B > 0 ? B : 0) * (T > 0 ? T : 0), Dh, M) : 0;
    case KVZAP_CALL_COMPRESS: {
      if (check_scorer_shape(Dh, M, H) != KVZAP_OK || (long long)B * H > 65535) return 0;
      const size_t a = M > 0 ? kvzap::score_mlp_workspace_bytes((long long)(B > 0 ? B : 0) * (T > 0 ? T : 0), Dh, M) : 0;
      const size_t b = mask_workspace(B, H, T);
      return a > b ? a : b;
    }
    case KVZAP_CALL_MASK_COMPACT:
      if ((long long)B * H > 65535) return 0;
      return mask_workspace(B, H, T);
    case KVZAP_CALL_ATTEND_DECODE:   // T = max_rows, Dh = HQ, M = window
      if (check_attend_shape(B, H, Dh, T, M) != KVZAP_OK) return 0;
      return kvzap::attend_workspace_bytes(B, H, Dh, T, M);
    case KVZAP_CALL_TEACHER_SCORES:       // T = prompt length, Dh = HQ, M = Tq
      if (Dh <= 0 || M <= 0 || Dh % H != 0 || H > 65535) return 0;
      return kvzap::teacher_workspace_bytes(H, Dh, M, T);
    case KVZAP_CALL_TOPK_THRESHOLD:
      if ((long long)B * H > 65535) return 0;
      return kvzap::topk_workspace_bytes(B, H, T, M != 0);
    case KVZAP_CALL_ASSIGN_PAGES:
      if ((long long)B * H > 65535) return 0;
      return kvzap::assign_pages_workspace_bytes(B * H);
    case KVZAP_CALL_COMPACT:
    default:
      return 0;
  }
}

namespace {
// argument checks of kvzap_score / kvzap_mask / kvzap_compact, shared with kvzap_compress
int check_score(const void* hidden, const void* W1, const void* b1, const void* W2,
                const void* b2, const float* scores, int B, int T, int Dh, int M, int H,
                const void* workspace, size_t workspace_bytes) {
  if (B < 0 || T < 0) return KVZAP_ERR_SHAPE;
  const int rc = check_scorer_shape(Dh, M, H);
  if (rc != KVZAP_OK) return rc;
  if ((long long)B * T > (long long)INT_MAX * 64) return KVZAP_ERR_SHAPE;
  if ((long long)B * T == 0) return KVZAP_OK;
  if (!hidden || !W1 || !scores) return KVZAP_ERR_NULL;
  if (M > 0 && !W2) return KVZAP_ERR_NULL;
  if (M == 0 && (W2 || b2)) return KVZAP_ERR_SHAPE;
  if (!aligned16(hidden) || !aligned16(W1) || !aligned16(scores) || !aligned16(W2) ||
      !aligned16(b1) || !aligned16(b2))
    return KVZAP_ERR_ALIGN;
  if (M > 0) {
    const size_t need = kvzap::score_mlp_workspace_bytes((long long)B * T, Dh, M);
    if (!workspace || !aligned256(workspace) || workspace_bytes < need) return KVZAP_ERR_WORKSPACE;
  }
  return KVZAP_OK;
}

int check_mask(const float* scores, float tau, int window, const int32_t* seq_lens, int B, int H,
               int T, const int32_t* keep_idx, const int32_t* lengths, const int64_t* offsets,
               const void* workspace, size_t workspace_bytes) {
  if (B <= 0 || H <= 0 || T <= 0 || window < 0) return KVZAP_ERR_SHAPE;
  if (tau != tau) return KVZAP_ERR_SHAPE;                 // NaN threshold
  if ((long long)B * H > 65535 || T > kMaxT) return KVZAP_ERR_UNSUPPORTED;
  if (!scores || !keep_idx || !lengths || !offsets) return KVZAP_ERR_NULL;
  if (!aligned16(scores) || !aligned16(keep_idx) || !aligned16(lengths) ||
      !aligned16(offsets) || !aligned16(seq_lens))
    return KVZAP_ERR_ALIGN;
  if (!workspace || !aligned256(workspace) || workspace_bytes < mask_workspace(B, H, T))
    return KVZAP_ERR_WORKSPACE;
  return KVZAP_OK;
}

int check_compact(const void* K, const void* V, const int32_t* keep_idx, const int32_t* lengths,
                  const int64_t* offsets, const void* K_out, const void* V_out, int64_t cap_rows,
                  int B, int H, int T, int D) {
  if (B <= 0 || H <= 0 || T <= 0 || D <= 0 || cap_rows < 0) return KVZAP_ERR_SHAPE;
  if (D % 8 != 0 || D > kMaxD || (long long)B * H > 65535 || T > kMaxT) return KVZAP_ERR_UNSUPPORTED;
  if (!K || !V || !keep_idx || !lengths || !offsets || !K_out || !V_out) return KVZAP_ERR_NULL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(keep_idx) || !aligned16(lengths) ||
      !aligned16(offsets) || !aligned16(K_out) || !aligned16(V_out))
    return KVZAP_ERR_ALIGN;
  // the gather is not an in-place operation
  const size_t in_bytes = (size_t)B * H * T * D * 2, out_bytes = (size_t)cap_rows * D * 2;
  auto overlaps = [](const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
  };
  if (overlaps(K, in_bytes, K_out, out_bytes) || overlaps(V, in_bytes, K_out, out_bytes) ||
      overlaps(K, in_bytes, V_out, out_bytes) || overlaps(V, in_bytes, V_out, out_bytes) ||
      overlaps(K_out, out_bytes, V_out, out_bytes))
    return KVZAP_ERR_SHAPE;
  return KVZAP_OK;
}

int run_score(const void* hidden, const void* W1, const void* b1, const void* W2, const void* b2,
              float* scores, int B, int T, int Dh, int M, int H, void* workspace, hipStream_t s) {
  if ((long long)B * T == 0) return KVZAP_OK;
  if (M > 0)
    return kvzap::launch_score_mlp(hidden, W1, b1, W2, b2, scores, B, T, Dh, M, H, workspace, s);
  return kvzap::launch_score_linear(hidden, W1, b1, scores, B, T, Dh, H, s);
}
}  // namespace

int kvzap_score(const void* hidden, const void* W1, const void* b1, const void* W2,
                const void* b2, float* scores, int B, int T, int Dh, int M, int H,
                void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_score(hidden, W1, b1, W2, b2, scores, B, T, Dh, M, H, workspace,
                             workspace_bytes);
  if (rc != KVZAP_OK) return rc;
  return run_score(hidden, W1, b1, W2, b2, scores, B, T, Dh, M, H, workspace,
                   static_cast<hipStream_t>(stream));
}

int kvzap_prepare_scorer(const void* W1, int Dh, int M, void* W1_prepared, size_t prepared_bytes,
                         void* stream) {
  const int rc = check_scorer_shape(Dh, M, 1);
  if (rc != KVZAP_OK) return rc;
  if (M == 0) return KVZAP_ERR_SHAPE;                     // the linear surrogate needs no preparation
  if (!W1 || !W1_prepared) return KVZAP_ERR_NULL;
  if (!aligned16(W1) || !aligned256(W1_prepared)) return KVZAP_ERR_ALIGN;
  if (prepared_bytes < kvzap::align_up((size_t)M * Dh * 2, 256)) return KVZAP_ERR_WORKSPACE;
  const size_t n = (size_t)M * Dh * 2;
  const uintptr_t a = reinterpret_cast<uintptr_t>(W1), b = reinterpret_cast<uintptr_t>(W1_prepared);
  if (a < b + n && b < a + n) return KVZAP_ERR_SHAPE;     // not an in-place operation
  return kvzap::launch_prepare_w1(W1, nullptr, Dh, M, W1_prepared, static_cast<hipStream_t>(stream));
}

int kvzap_prepare_scorer_rmsnorm(const void* W1, const void* gain, int Dh, int M,
                                 void* W1_prepared, size_t prepared_bytes, void* stream) {
  const int rc = check_scorer_shape(Dh, M, 1);
  if (rc != KVZAP_OK) return rc;
  if (M == 0) return KVZAP_ERR_SHAPE;
  if (!kvzap::score_rmsnorm_supports(Dh)) return KVZAP_ERR_UNSUPPORTED;
  if (!W1 || !gain || !W1_prepared) return KVZAP_ERR_NULL;
  if (!aligned16(W1) || !aligned16(gain) || !aligned256(W1_prepared)) return KVZAP_ERR_ALIGN;
  if (prepared_bytes < kvzap::align_up((size_t)M * Dh * 2, 256)) return KVZAP_ERR_WORKSPACE;
  const size_t n = (size_t)M * Dh * 2;
  const uintptr_t a = reinterpret_cast<uintptr_t>(W1), b = reinterpret_cast<uintptr_t>(W1_prepared);
  if (a < b + n && b < a + n) return KVZAP_ERR_SHAPE;     // not an in-place operation
  return kvzap::launch_prepare_w1(W1, gain, Dh, M, W1_prepared, static_cast<hipStream_t>(stream));
}

int kvzap_score_rmsnorm(const void* x, const void* W1_prepared, const void* gain, float eps,
                        const void* b1, const void* W2, const void* b2, float* scores,
                        float* rstd, void* normed, int B, int T, int Dh, int M, int H,
                        void* stream) {
  if (M <= 0) return M == 0 ? KVZAP_ERR_UNSUPPORTED : KVZAP_ERR_SHAPE;   // MLP surrogate only
  if (!(eps >= 0.0f)) return KVZAP_ERR_SHAPE;                          // also NaN
  int rc = check_score(x, W1_prepared, b1, W2, b2, scores, B, T, Dh, M, H, W1_prepared, ~(size_t)0);
  if (rc != KVZAP_OK) return rc == KVZAP_ERR_WORKSPACE ? KVZAP_ERR_ALIGN : rc;
  if (!kvzap::score_rmsnorm_supports(Dh)) return KVZAP_ERR_UNSUPPORTED;
  if ((long long)B * T == 0) return KVZAP_OK;
  if (!gain || !rstd) return KVZAP_ERR_NULL;
  if (!aligned16(gain) || !aligned16(rstd) || !aligned16(normed)) return KVZAP_ERR_ALIGN;
  if (normed) {                                                        // not an in-place operation
    const size_t n = (size_t)B * T * Dh * 2;
    const uintptr_t a = reinterpret_cast<uintptr_t>(x), b = reinterpret_cast<uintptr_t>(normed);
    if (a < b + n && b < a + n) return KVZAP_ERR_SHAPE;
  }
  return kvzap::launch_score_mlp_rmsnorm(x, W1_prepared, gain, eps, b1, W2, b2, scores, rstd, normed,
                                         B, T, Dh, M, H, static_cast<hipStream_t>(stream));
}

int kvzap_score_prepared(const void* hidden, const void* W1_prepared, const void* b1,
                         const void* W2, const void* b2, float* scores, int B, int T, int Dh,
                         int M, int H, void* stream) {
  if (M <= 0) return KVZAP_ERR_SHAPE;
  // as kvzap_score, with the workspace requirement replaced by the prepared copy's alignment
  int rc = check_score(hidden, W1_prepared, b1, W2, b2, scores, B, T, Dh, M, H,
                       W1_prepared, ~(size_t)0);
  if (rc != KVZAP_OK) return rc == KVZAP_ERR_WORKSPACE ? KVZAP_ERR_ALIGN : rc;
  if ((long long)B * T == 0) return KVZAP_OK;
  return kvzap::launch_score_mlp(hidden, W1_prepared, b1, W2, b2, scores, B, T, Dh, M, H, nullptr,
                                 static_cast<hipStream_t>(stream));
}

int kvzap_mask(const float* scores, float tau, int window, const int32_t* seq_lens, int B,
               int H, int T, int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
               void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_mask(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets,
                            workspace, workspace_bytes);
  if (rc != KVZAP_OK) return rc;
  return kvzap::launch_mask(scores, tau, nullptr, window, seq_lens, B, H, T, keep_idx, lengths,
                            offsets, workspace, static_cast<hipStream_t>(stream));
}

int kvzap_mask_static(const float* scores, float tau, int window, const int32_t* seq_lens, int B,
                      int H, int T, int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                      void* stream) {
  // kvzap_mask's checks, the workspace ones aside (the scratch is the library's own)
  const int rc = check_mask(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets,
                            reinterpret_cast<const void*>(uintptr_t{256}), ~(size_t)0);
  if (rc != KVZAP_OK) return rc;
  return kvzap::launch_mask_static(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths,
                                   offsets, static_cast<hipStream_t>(stream));
}

int kvzap_mask_per_head(const float* scores, const float* tau, int window,
                        const int32_t* seq_lens, int B, int H, int T, int32_t* keep_idx,
                        int32_t* lengths, int64_t* offsets, void* workspace,
                        size_t workspace_bytes, void* stream) {
  if (B <= 0 || H <= 0 || T <= 0 || window < 0) return KVZAP_ERR_SHAPE;
  if ((long long)B * H > 65535 || T > kMaxT) return KVZAP_ERR_UNSUPPORTED;
  if (!scores || !tau || !keep_idx || !lengths || !offsets) return KVZAP_ERR_NULL;
  if (!aligned16(scores) || !aligned16(tau) || !aligned16(keep_idx) || !aligned16(lengths) ||
      !aligned16(offsets) || !aligned16(seq_lens))
    return KVZAP_ERR_ALIGN;
  if (!workspace || !aligned256(workspace) || workspace_bytes < mask_workspace(B, H, T))
    return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_mask(scores, 0.0f, tau, window, seq_lens, B, H, T, keep_idx, lengths,
                            offsets, workspace, static_cast<hipStream_t>(stream));
}

int kvzap_topk_threshold(const float* scores, int window, const int32_t* seq_lens, int64_t k,
                         int per_layer, int B, int H, int T, float* tau_out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (B <= 0 || H <= 0 || T <= 0 || window < 0) return KVZAP_ERR_SHAPE;
  if ((long long)B * H > 65535 || T > kMaxT) return KVZAP_ERR_UNSUPPORTED;
  if ((long long)H * T > 0xFFFFFFFFll) return KVZAP_ERR_UNSUPPORTED;     // 32-bit histogram bins
  if (!scores || !tau_out) return KVZAP_ERR_NULL;
  if (!aligned16(scores) || !aligned16(tau_out) || !aligned16(seq_lens)) return KVZAP_ERR_ALIGN;
  if (!workspace || !aligned256(workspace) ||
      workspace_bytes < kvzap::topk_workspace_bytes(B, H, T, per_layer != 0))
    return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_topk_threshold(scores, window, seq_lens, (long long)k, per_layer != 0, B,
                                      H, T, tau_out, workspace, static_cast<hipStream_t>(stream));
}

int kvzap_compact(const void* K, const void* V, const int32_t* keep_idx,
                  const int32_t* lengths, const int64_t* offsets, void* K_out, void* V_out,
                  int64_t cap_rows, int B, int H, int T, int D, void* stream) {
  const int rc = check_compact(K, V, keep_idx, lengths, offsets, K_out, V_out, cap_rows, B, H, T, D);
  if (rc != KVZAP_OK) return rc;
  return kvzap::launch_compact(K, V, keep_idx, lengths, offsets, K_out, V_out, cap_rows, B * H,
                               T, D, static_cast<hipStream_t>(stream));
}

namespace {
// threshold + gather on given scores (all arguments checked)
int run_mask_compact(const float* scores, float tau, int window, const int32_t* seq_lens, int B,
                     int H, int T, int32_t* keep_idx, int32_t* lengths, int64_t* offsets,
                     const void* K, const void* V, void* K_out, void* V_out, int64_t cap_rows, int D,
                     void* workspace, hipStream_t s) {
  const int rc = kvzap::launch_mask(scores, tau, nullptr, window, seq_lens, B, H, T, keep_idx,
                                    lengths, offsets, workspace, s);
  if (rc != KVZAP_OK) return rc;
  return kvzap::launch_compact(K, V, keep_idx, lengths, offsets, K_out, V_out, cap_rows, B * H, T,
                               D, s);
}
}  // namespace

int kvzap_mask_compact(const float* scores, float tau, int window, const int32_t* seq_lens,
                       const void* K, const void* V, int32_t* keep_idx, int32_t* lengths,
                       int64_t* offsets, void* K_out, void* V_out, int64_t cap_rows, int B, int H,
                       int T, int D, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_mask(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets, workspace,
                      workspace_bytes);
  if (rc == KVZAP_OK)
    rc = check_compact(K, V, keep_idx, lengths, offsets, K_out, V_out, cap_rows, B, H, T, D);
  if (rc != KVZAP_OK) return rc;
  return run_mask_compact(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets, K, V,
                          K_out, V_out, cap_rows, D, workspace, static_cast<hipStream_t>(stream));
}

int kvzap_compress(const void* hidden, const void* W1, const void* b1, const void* W2,
                   const void* b2, const void* K, const void* V, float tau, int window,
                   const int32_t* seq_lens, float* scores, int32_t* keep_idx, int32_t* lengths,
                   int64_t* offsets, void* K_out, void* V_out, int64_t cap_rows, int B, int T,
                   int Dh, int M, int H, int D, void* workspace, size_t workspace_bytes,
                   void* stream) {
  // all three sets of checks before anything is launched (the mask's demand B, T > 0)
  int rc = check_mask(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets, workspace,
                      workspace_bytes);
  if (rc == KVZAP_OK)
    rc = check_score(hidden, W1, b1, W2, b2, scores, B, T, Dh, M, H, workspace, workspace_bytes);
  if (rc == KVZAP_OK)
    rc = check_compact(K, V, keep_idx, lengths, offsets, K_out, V_out, cap_rows, B, H, T, D);
  if (rc != KVZAP_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the score workspace (W1 in fragment order) is dead once the scorer has run, the mask
  // then reuses the same bytes on the same stream
  rc = run_score(hidden, W1, b1, W2, b2, scores, B, T, Dh, M, H, workspace, s);
  if (rc != KVZAP_OK) return rc;
  return run_mask_compact(scores, tau, window, seq_lens, B, H, T, keep_idx, lengths, offsets, K, V,
                          K_out, V_out, cap_rows, D, workspace, s);
}

int kvzap_decode_evict(const void* hidden_new, const void* W1, const void* b1, const void* W2,
                       const void* b2, int Dh, int M, const void* k_new, const void* v_new,
                       void* K_prefix, void* V_prefix, int32_t* prefix_pos,
                       const int64_t* slab_offsets, const int32_t* slab_capacity, void* K_ring,
                       void* V_ring, float* score_ring, int32_t* lengths, int32_t* seq_pos,
                       float tau, int window, int B, int H, int D, int32_t* error_flag,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (B <= 0 || H <= 0 || D <= 0 || window < 0) return KVZAP_ERR_SHAPE;
  if (tau != tau) return KVZAP_ERR_SHAPE;
  const int rc = check_scorer_shape(Dh, M, H);
  if (rc != KVZAP_OK) return rc;
  if (D % 8 != 0 || D > kMaxD || B > 65535) return KVZAP_ERR_UNSUPPORTED;
  if (!hidden_new || !W1 || !k_new || !v_new || !K_prefix || !V_prefix || !prefix_pos ||
      !slab_offsets || !slab_capacity || !lengths || !seq_pos)
    return KVZAP_ERR_NULL;
  if (window > 0 && (!K_ring || !V_ring || !score_ring)) return KVZAP_ERR_NULL;
  if (M > 0 && !W2) return KVZAP_ERR_NULL;
  if (M == 0 && (W2 || b2)) return KVZAP_ERR_SHAPE;
  const void* ptrs[] = {hidden_new, W1, b1, W2, b2, k_new, v_new, K_prefix, V_prefix,
                        prefix_pos, slab_offsets, slab_capacity, K_ring, V_ring, score_ring,
                        lengths, seq_pos};
  for (const void* p : ptrs)
    if (!aligned16(p)) return KVZAP_ERR_ALIGN;
  const size_t need = kvzap::decode_workspace_bytes(B, Dh, M, H);
  if (need > 0 && (!workspace || !aligned256(workspace) || workspace_bytes < need))
    return KVZAP_ERR_WORKSPACE;
  kvzap::DecodeArgs a;
  a.hidden_new = hidden_new; a.W1 = W1; a.b1 = b1; a.W2 = W2; a.b2 = b2;
  a.Dh = Dh; a.M = M; a.k_new = k_new; a.v_new = v_new;
  a.K_prefix = K_prefix; a.V_prefix = V_prefix; a.prefix_pos = prefix_pos;
  a.slab_offsets = slab_offsets; a.slab_capacity = slab_capacity;
  a.K_ring = K_ring; a.V_ring = V_ring; a.score_ring = score_ring;
  a.lengths = lengths; a.seq_pos = seq_pos; a.tau = tau; a.window = window;
  a.B = B; a.H = H; a.D = D; a.error_flag = error_flag; a.workspace = workspace;
  a.block_table = nullptr; a.max_pages = 0; a.log_page = 0; a.num_pages = 0;
  return kvzap::launch_decode_evict(a, static_cast<hipStream_t>(stream));
}

int kvzap_attend_decode(const void* q, const void* K_rows, const void* V_rows,
                        int64_t total_rows, const int64_t* row_offsets, const int32_t* lengths,
                        const void* K_ring, const void* V_ring, const int32_t* seq_pos,
                        int window, int max_rows, float scale, void* out, int B, int H, int HQ,
                        int D, void* workspace, size_t workspace_bytes, void* stream) {
  if (D <= 0 || total_rows < 0) return KVZAP_ERR_SHAPE;
  const int rc = check_attend_shape(B, H, HQ, max_rows, window);
  if (rc != KVZAP_OK) return rc;
  if (D != 128) return KVZAP_ERR_UNSUPPORTED;
  if (scale != scale) return KVZAP_ERR_SHAPE;
  if (!q || !row_offsets || !lengths || !out) return KVZAP_ERR_NULL;
  if (total_rows > 0 && (!K_rows || !V_rows)) return KVZAP_ERR_NULL;
  if (window > 0 && (!K_ring || !V_ring || !seq_pos)) return KVZAP_ERR_NULL;
  const void* ptrs[] = {q, K_rows, V_rows, row_offsets, lengths, K_ring, V_ring, seq_pos, out};
  for (const void* p : ptrs)
    if (!aligned16(p)) return KVZAP_ERR_ALIGN;
  const size_t need = kvzap::attend_workspace_bytes(B, H, HQ, max_rows, window);
  if (!workspace || !aligned256(workspace) || workspace_bytes < need) return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_attend_decode(q, K_rows, V_rows, total_rows, row_offsets, nullptr, 0, 0, 0,
                                     lengths, K_ring, V_ring, seq_pos, window, max_rows, scale,
                                     out, B, H, HQ, workspace, static_cast<hipStream_t>(stream));
}

namespace {
bool valid_page_rows(int page_rows) {
  return page_rows >= 16 && page_rows <= (1 << 20) && (page_rows & (page_rows - 1)) == 0;
}
}  // namespace

int kvzap_assign_pages(const int32_t* lengths, int B, int H, int page_rows, int reserve_rows,
                       const int32_t* free_pages, int n_free, int32_t* block_table,
                       int max_pages, int32_t* result, void* workspace, size_t workspace_bytes,
                       void* stream) {
  if (B <= 0 || H <= 0 || reserve_rows < 0 || n_free < 0 || max_pages <= 0) return KVZAP_ERR_SHAPE;
  if (!valid_page_rows(page_rows)) return KVZAP_ERR_SHAPE;
  if ((long long)B * H > 65535) return KVZAP_ERR_UNSUPPORTED;
  if (!lengths || !block_table || !result || (n_free > 0 && !free_pages)) return KVZAP_ERR_NULL;
  if (!aligned16(lengths) || !aligned4(free_pages) || !aligned16(block_table) || !aligned16(result))
    return KVZAP_ERR_ALIGN;
  if (!workspace || !aligned256(workspace) ||
      workspace_bytes < kvzap::assign_pages_workspace_bytes(B * H))
    return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_assign_pages(lengths, nullptr, B * H, page_rows, reserve_rows, free_pages,
                                    n_free, block_table, max_pages, result, workspace,
                                    static_cast<hipStream_t>(stream));
}

int kvzap_extend_pages(const int32_t* lengths, int32_t* page_counts, int B, int H, int page_rows,
                       int reserve_rows, const int32_t* free_pages, int n_free,
                       int32_t* block_table, int max_pages, int32_t* result, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (B <= 0 || H <= 0 || reserve_rows < 0 || n_free < 0 || max_pages <= 0) return KVZAP_ERR_SHAPE;
  if (!valid_page_rows(page_rows)) return KVZAP_ERR_SHAPE;
  if ((long long)B * H > 65535) return KVZAP_ERR_UNSUPPORTED;
  if (!lengths || !page_counts || !block_table || !result || (n_free > 0 && !free_pages))
    return KVZAP_ERR_NULL;
  if (!aligned16(lengths) || !aligned16(page_counts) || !aligned4(free_pages) ||
      !aligned16(block_table) || !aligned16(result))
    return KVZAP_ERR_ALIGN;
  if (!workspace || !aligned256(workspace) ||
      workspace_bytes < kvzap::assign_pages_workspace_bytes(B * H))
    return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_assign_pages(lengths, page_counts, B * H, page_rows, reserve_rows,
                                    free_pages, n_free, block_table, max_pages, result, workspace,
                                    static_cast<hipStream_t>(stream));
}

int kvzap_decode_evict_paged(const void* hidden_new, const void* W1, const void* b1,
                             const void* W2, const void* b2, int Dh, int M, const void* k_new,
                             const void* v_new, void* K_pool, void* V_pool, int32_t* pos_pool,
                             int num_pages, const int32_t* block_table, int max_pages,
                             int page_rows, void* K_ring, void* V_ring, float* score_ring,
                             int32_t* lengths, int32_t* seq_pos, float tau, int window, int B,
                             int H, int D, int32_t* error_flag, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (B <= 0 || H <= 0 || D <= 0 || window < 0 || num_pages < 0 || max_pages <= 0)
    return KVZAP_ERR_SHAPE;
  if (!valid_page_rows(page_rows) || tau != tau) return KVZAP_ERR_SHAPE;
  const int rc = check_scorer_shape(Dh, M, H);
  if (rc != KVZAP_OK) return rc;
  if (D % 8 != 0 || D > kMaxD || B > 65535) return KVZAP_ERR_UNSUPPORTED;
  if (!hidden_new || !W1 || !k_new || !v_new || !block_table || !lengths || !seq_pos)
    return KVZAP_ERR_NULL;
  if (num_pages > 0 && (!K_pool || !V_pool || !pos_pool)) return KVZAP_ERR_NULL;
  if (window > 0 && (!K_ring || !V_ring || !score_ring)) return KVZAP_ERR_NULL;
  if (M > 0 && !W2) return KVZAP_ERR_NULL;
  if (M == 0 && (W2 || b2)) return KVZAP_ERR_SHAPE;
  const void* ptrs[] = {hidden_new, W1, b1, W2, b2, k_new, v_new, K_pool, V_pool, pos_pool,
                        block_table, K_ring, V_ring, score_ring, lengths, seq_pos};
  for (const void* p : ptrs)
    if (!aligned16(p)) return KVZAP_ERR_ALIGN;
  const size_t need = kvzap::decode_workspace_bytes(B, Dh, M, H);
  if (need > 0 && (!workspace || !aligned256(workspace) || workspace_bytes < need))
    return KVZAP_ERR_WORKSPACE;
  kvzap::DecodeArgs a;
  a.hidden_new = hidden_new; a.W1 = W1; a.b1 = b1; a.W2 = W2; a.b2 = b2;
  a.Dh = Dh; a.M = M; a.k_new = k_new; a.v_new = v_new;
  a.K_prefix = K_pool; a.V_prefix = V_pool; a.prefix_pos = pos_pool;
  a.slab_offsets = nullptr; a.slab_capacity = nullptr;
  a.K_ring = K_ring; a.V_ring = V_ring; a.score_ring = score_ring;
  a.lengths = lengths; a.seq_pos = seq_pos; a.tau = tau; a.window = window;
  a.B = B; a.H = H; a.D = D; a.error_flag = error_flag; a.workspace = workspace;
  a.block_table = block_table; a.max_pages = max_pages; a.num_pages = num_pages;
  a.log_page = 0;
  while ((1 << a.log_page) < page_rows) ++a.log_page;
  return kvzap::launch_decode_evict(a, static_cast<hipStream_t>(stream));
}

int kvzap_compact_paged(const void* K, const void* V, const int32_t* keep_idx,
                        const int32_t* lengths, const int64_t* offsets,
                        const int32_t* block_table, int max_pages, int page_rows, void* K_pool,
                        void* V_pool, int num_pages, int B, int H, int T, int D, void* stream) {
  if (B <= 0 || H <= 0 || T <= 0 || D <= 0 || max_pages <= 0 || num_pages < 0) return KVZAP_ERR_SHAPE;
  if (!valid_page_rows(page_rows)) return KVZAP_ERR_SHAPE;
  if ((D != 64 && D != 128 && D != 256) || (long long)B * H > 65535 || T > kMaxT) return KVZAP_ERR_UNSUPPORTED;
  if (!K || !V || !keep_idx || !lengths || !offsets || !block_table) return KVZAP_ERR_NULL;
  if (num_pages > 0 && (!K_pool || !V_pool)) return KVZAP_ERR_NULL;
  const void* ptrs[] = {K, V, keep_idx, lengths, offsets, block_table, K_pool, V_pool};
  for (const void* p : ptrs)
    if (!aligned16(p)) return KVZAP_ERR_ALIGN;
  {  // the gather is not an in-place operation
    const size_t in_bytes = (size_t)B * H * T * D * 2;
    const size_t pool_bytes = (size_t)num_pages * page_rows * D * 2;
    auto overlaps = [](const void* a, size_t na, const void* b, size_t nb) {
      const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
      return na > 0 && nb > 0 && x < y + nb && y < x + na;
    };
    if (overlaps(K, in_bytes, K_pool, pool_bytes) || overlaps(V, in_bytes, K_pool, pool_bytes) ||
        overlaps(K, in_bytes, V_pool, pool_bytes) || overlaps(V, in_bytes, V_pool, pool_bytes) ||
        overlaps(K_pool, pool_bytes, V_pool, pool_bytes))
      return KVZAP_ERR_SHAPE;
  }
  if (num_pages == 0) return KVZAP_OK;                   // nothing can be written
  return kvzap::launch_compact_paged(K, V, keep_idx, lengths, offsets, block_table, max_pages,
                                     page_rows, K_pool, V_pool, num_pages, B * H, T, D,
                                     static_cast<hipStream_t>(stream));
}

int kvzap_attend_decode_paged(const void* q, const void* K_pool, const void* V_pool,
                              int num_pages, const int32_t* block_table, int max_pages,
                              int page_rows, const int32_t* lengths, const void* K_ring,
                              const void* V_ring, const int32_t* seq_pos, int window,
                              int max_rows, float scale, void* out, int B, int H, int HQ, int D,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (D <= 0 || num_pages < 0 || max_pages <= 0) return KVZAP_ERR_SHAPE;
  if (!valid_page_rows(page_rows)) return KVZAP_ERR_SHAPE;
  const int rc = check_attend_shape(B, H, HQ, max_rows, window);
  if (rc != KVZAP_OK) return rc;
  if (D != 128) return KVZAP_ERR_UNSUPPORTED;
  if (scale != scale) return KVZAP_ERR_SHAPE;
  if ((long long)max_pages * page_rows > INT_MAX) return KVZAP_ERR_SHAPE;
  if (!q || !block_table || !lengths || !out) return KVZAP_ERR_NULL;
  if (num_pages > 0 && (!K_pool || !V_pool)) return KVZAP_ERR_NULL;
  if (window > 0 && (!K_ring || !V_ring || !seq_pos)) return KVZAP_ERR_NULL;
  const void* ptrs[] = {q, K_pool, V_pool, block_table, lengths, K_ring, V_ring, seq_pos, out};
  for (const void* p : ptrs)
    if (!aligned16(p)) return KVZAP_ERR_ALIGN;
  const size_t need = kvzap::attend_workspace_bytes(B, H, HQ, max_rows, window);
  if (!workspace || !aligned256(workspace) || workspace_bytes < need) return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_attend_decode(q, K_pool, V_pool, 0, nullptr, block_table, max_pages,
                                     page_rows, num_pages, lengths, K_ring, V_ring, seq_pos, window,
                                     max_rows, scale, out, B, H, HQ, workspace,
                                     static_cast<hipStream_t>(stream));
}

int kvzap_teacher_scores(const void* q, const void* k, const float* vnorm, const float* hnorm,
                         float scale, float* log_s, int H, int HQ, int Tq, int Tk, int T, int D,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (H <= 0 || HQ <= 0 || Tq <= 0 || Tk < Tq || T < 0 || D <= 0) return KVZAP_ERR_SHAPE;
  if (HQ % H != 0 || T > Tk - Tq || !(scale > 0.0f)) return KVZAP_ERR_SHAPE;   // also NaN
  if (D != 128 || H > 65535 || HQ > 65535 || (long long)Tk > (1ll << 30)) return KVZAP_ERR_UNSUPPORTED;
  if (!q || !k || (T > 0 && !log_s)) return KVZAP_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(vnorm) || !aligned16(hnorm) || !aligned16(log_s))
    return KVZAP_ERR_ALIGN;
  if (T == 0) return KVZAP_OK;                              // nothing to score
  if (!workspace || !aligned256(workspace) ||
      workspace_bytes < kvzap::teacher_workspace_bytes(H, HQ, Tq, T))
    return KVZAP_ERR_WORKSPACE;
  return kvzap::launch_teacher_scores(q, k, vnorm, hnorm, scale, log_s, H, HQ, Tq, Tk, T, workspace,
                                      static_cast<hipStream_t>(stream));
}

}  // extern "C"
