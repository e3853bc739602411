// C ABI of libcopris: argument checks on the host, then kernel launches on the
// caller's stream.  No allocation, no synchronisation, no host copies.
#include "copris.h"
#include "copris_internal.h"

#include <cstdio>

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

thread_local char g_detail[256] = "";
copris_launch_hook_fn g_hook = nullptr;
void* g_hook_user = nullptr;

bool attn_shape_ok(int C, int Hq, int Hkv, int D, int page_size, int max_pages) {
  if (C <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || max_pages <= 0) return false;
  if (Hq % Hkv != 0) return false;
  if (static_cast<int64_t>(max_pages) * page_size > (1ll << 30)) return false;
  if (static_cast<int64_t>(C) * Hkv >= (1ll << 20)) return false;
  // the generic path indexes (sequence, 512-token chunk, kv head) items with 32 bits
  const int64_t chunks = (static_cast<int64_t>(max_pages) * page_size + copris::kAttnChunkTokens - 1) /
                         copris::kAttnChunkTokens;
  if (static_cast<int64_t>(C) * chunks * Hkv >= (1ll << 31)) return false;
  return true;
}

bool attn_supported(int Hq, int Hkv, int D, int page_size, int dtype) {
  if (dtype != COPRIS_F32 && dtype != COPRIS_BF16) return false;
  if (D != 64 && D != 128) return false;
  if (Hq / Hkv > copris::kAttnMaxGroup) return false;
  // a split-K chunk must hold whole pages
  if (page_size > copris::kAttnChunkTokens || copris::kAttnChunkTokens % page_size != 0) return false;
  return true;
}

}  // namespace

namespace copris {
bool launch_ok(const char* kernel_name) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return true;
  snprintf(g_detail, sizeof(g_detail), "%s: %s (%s)", kernel_name, hipGetErrorName(e),
           hipGetErrorString(e));
  return false;
}
void set_error_detail(const char* what, hipError_t e) {
  snprintf(g_detail, sizeof(g_detail), "%s: %s (%s)", what, hipGetErrorName(e), hipGetErrorString(e));
}
void launch_hook(const char* kernel_name, int phase, hipStream_t stream) {
  if (g_hook != nullptr) g_hook(kernel_name, phase, static_cast<void*>(stream), g_hook_user);
}
}  // namespace copris

extern "C" {

const char* copris_strerror(int code) {
  switch (code) {
    case COPRIS_OK: return "ok";
    case COPRIS_EINVAL: return "invalid argument (null pointer, bad shape, misaligned base or bad scalar)";
    case COPRIS_EWORKSPACE: return "workspace too small or misaligned";
    case COPRIS_EUNSUPPORTED: return "unsupported dtype / head_dim / page_size / group size";
    case COPRIS_ELAUNCH: return "HIP runtime error at kernel launch";
    default: return "unknown error code";
  }
}

const char* copris_version(void) { return "0.1.0"; }

const char* copris_last_error_detail(void) { return g_detail; }

void copris_set_launch_hook(copris_launch_hook_fn hook, void* user) {
  g_hook = hook;
  g_hook_user = user;
}

size_t copris_decode_attn_workspace_bytes(int C, int Hq, int Hkv, int D, int page_size,
                                          int max_pages) {
  if (!attn_shape_ok(C, Hq, Hkv, D, page_size, max_pages)) return 0;
  return copris::attn_workspace_layout(C, Hq, Hkv, D, page_size, max_pages).total;
}

int copris_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_len, void* out, float* lse,
                       void* workspace, size_t workspace_bytes, int C, int Hq, int Hkv, int D,
                       int page_size, int max_pages, int64_t num_pages, float scale, int dtype,
                       void* stream) {
  if (!q || !k_cache || !v_cache || !block_table || !ctx_len || !out || !workspace)
    return COPRIS_EINVAL;
  if (!attn_shape_ok(C, Hq, Hkv, D, page_size, max_pages) || num_pages <= 0) return COPRIS_EINVAL;
  if (!(scale > 0.0f) || !(scale < INFINITY)) return COPRIS_EINVAL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      !aligned16(block_table) || !aligned16(ctx_len) || (lse && !aligned16(lse)))
    return COPRIS_EINVAL;
  if (!attn_supported(Hq, Hkv, D, page_size, dtype)) return COPRIS_EUNSUPPORTED;
  if (!aligned256(workspace) ||
      workspace_bytes < copris_decode_attn_workspace_bytes(C, Hq, Hkv, D, page_size, max_pages))
    return COPRIS_EWORKSPACE;
  (void)hipGetLastError();
  return copris::launch_decode_attn(q, k_cache, v_cache, block_table, ctx_len, out, lse, workspace, C, Hq,
                             Hkv, D, page_size, max_pages, scale, dtype,
                             static_cast<hipStream_t>(stream));
}

int copris_prefill_attn(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                        const int32_t* block_table, void* k_cache, void* v_cache, void* out,
                        float* lse, int B, int64_t T, int Hq, int Hkv, int D, int page_size,
                        int max_pages, int64_t num_pages, int max_seqlen, float scale, int dtype,
                        void* stream) {
  if (B < 0 || T < 0 || T >= (1ll << 31)) return COPRIS_EINVAL;
  if (B == 0 || T == 0) return (B == 0 && T != 0) ? COPRIS_EINVAL : COPRIS_OK;
  if (!q || !k || !v || !cu_seqlens || !block_table || !k_cache || !v_cache || !out)
    return COPRIS_EINVAL;
  if (Hq <= 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || max_pages <= 0 || num_pages <= 0 ||
      Hq % Hkv != 0 || Hkv > 65535 || B > 65535)
    return COPRIS_EINVAL;
  if (max_seqlen <= 0 || static_cast<int64_t>(max_seqlen) > static_cast<int64_t>(max_pages) * page_size)
    return COPRIS_EINVAL;
  if (!(scale > 0.0f) || !(scale < INFINITY)) return COPRIS_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache) ||
      !aligned16(out) || (lse && !aligned16(lse)))
    return COPRIS_EINVAL;
  if (!copris::prefill_attn_supported(Hq, Hkv, D, page_size, dtype)) return COPRIS_EUNSUPPORTED;
  (void)hipGetLastError();
  return copris::launch_prefill_attn(q, k, v, cu_seqlens, block_table, k_cache, v_cache, out, lse, B,
                                     Hq, Hkv, max_pages, max_seqlen, scale,
                                     static_cast<hipStream_t>(stream));
}

size_t copris_lmhead_logprob_workspace_bytes(int C, int H, int V) {
  if (C <= 0 || H <= 0 || V <= 0) return 0;
  return copris::lm_workspace_layout(C, H, V).total;
}

int copris_lmhead_logprob(const void* hidden, const void* weight, const int64_t* seq_id,
                          const int32_t* step, uint64_t seed, float temperature, int32_t* token,
                          float* logprob, float* lse, void* workspace, size_t workspace_bytes,
                          int C, int H, int V, int dtype, void* stream) {
  if (!hidden || !weight || !seq_id || !step || !token || !logprob || !workspace)
    return COPRIS_EINVAL;
  if (C <= 0 || H <= 0 || V <= 0) return COPRIS_EINVAL;
  if (!(temperature > 0.0f) || !(temperature < INFINITY)) return COPRIS_EINVAL;
  if (dtype != COPRIS_F32 && dtype != COPRIS_BF16) return COPRIS_EUNSUPPORTED;
  if (H % (dtype == COPRIS_BF16 ? 8 : 4) != 0) return COPRIS_EINVAL;
  if (!aligned16(hidden) || !aligned16(weight) || !aligned16(seq_id) || !aligned16(step) ||
      !aligned16(token) || !aligned16(logprob) || (lse && !aligned16(lse)))
    return COPRIS_EINVAL;
  if (!aligned256(workspace) || workspace_bytes < copris_lmhead_logprob_workspace_bytes(C, H, V))
    return COPRIS_EWORKSPACE;
  (void)hipGetLastError();
  return copris::launch_lmhead_logprob(hidden, weight, seq_id, step, seed, temperature, token, logprob,
                                lse, workspace, C, H, V, dtype, static_cast<hipStream_t>(stream));
}

int copris_lmhead_logprob_noalloc(const void* hidden, const void* weight, const int64_t* seq_id,
                                  const int32_t* step, uint64_t seed, float temperature,
                                  int32_t* token, float* logprob, float* lse, int C, int H, int V,
                                  int dtype, void* stream) {
  if (!hidden || !weight || !seq_id || !step || !token || !logprob) return COPRIS_EINVAL;
  if (C <= 0 || H <= 0 || V <= 0) return COPRIS_EINVAL;
  if (!(temperature > 0.0f) || !(temperature < INFINITY)) return COPRIS_EINVAL;
  if (dtype != COPRIS_F32 && dtype != COPRIS_BF16) return COPRIS_EUNSUPPORTED;
  if (H % (dtype == COPRIS_BF16 ? 8 : 4) != 0) return COPRIS_EINVAL;
  if (!aligned16(hidden) || !aligned16(weight) || !aligned16(seq_id) || !aligned16(step) ||
      !aligned16(token) || !aligned16(logprob) || (lse && !aligned16(lse)))
    return COPRIS_EINVAL;
  if (copris::lm_noalloc_scratch_needed(C, H, V, dtype) > copris::lm_noalloc_scratch_limit()) {
    snprintf(g_detail, sizeof(g_detail),
             "copris_lmhead_logprob_noalloc: C=%d H=%d V=%d needs %zu bytes of partials, the static "
             "array holds %zu", C, H, V, copris::lm_noalloc_scratch_needed(C, H, V, dtype),
             copris::lm_noalloc_scratch_limit());
    return COPRIS_EWORKSPACE;
  }
  (void)hipGetLastError();
  return copris::launch_lmhead_logprob_noalloc(hidden, weight, seq_id, step, seed, temperature, token,
                                               logprob, lse, C, H, V, dtype,
                                               static_cast<hipStream_t>(stream));
}

size_t copris_lmhead_logprob_noalloc_max_bytes(void) { return copris::lm_noalloc_scratch_limit(); }

size_t copris_lmhead_token_logprob_workspace_bytes(int M, int H, int V, int dtype) {
  if (M <= 0 || H <= 0 || V <= 0 || (dtype != COPRIS_F32 && dtype != COPRIS_BF16)) return 0;
  return copris::lm_token_workspace_bytes(M, H, V, dtype);
}

int copris_lmhead_token_logprob(const void* hidden, const void* weight, const int32_t* tokens,
                                float temperature, float* logprob, float* lse, void* workspace,
                                size_t workspace_bytes, int M, int H, int V, int dtype,
                                void* stream) {
  if (!hidden || !weight || !tokens || !logprob || !workspace) return COPRIS_EINVAL;
  if (M <= 0 || H <= 0 || V <= 0) return COPRIS_EINVAL;
  if (!(temperature > 0.0f) || !(temperature < INFINITY)) return COPRIS_EINVAL;
  if (dtype != COPRIS_F32 && dtype != COPRIS_BF16) return COPRIS_EUNSUPPORTED;
  if (H % (dtype == COPRIS_BF16 ? 8 : 4) != 0) return COPRIS_EINVAL;
  if (!aligned16(hidden) || !aligned16(weight) || !aligned16(tokens) || !aligned16(logprob) ||
      (lse && !aligned16(lse)))
    return COPRIS_EINVAL;
  if (!aligned256(workspace) ||
      workspace_bytes < copris_lmhead_token_logprob_workspace_bytes(M, H, V, dtype))
    return COPRIS_EWORKSPACE;
  (void)hipGetLastError();
  return copris::launch_lmhead_token_logprob(hidden, weight, tokens, temperature, logprob, lse,
                                             workspace, M, H, V, dtype,
                                             static_cast<hipStream_t>(stream));
}

int copris_is_ratio(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                    const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                    float eps_low, float eps_high, float* ratio, float* ratio_clipped,
                    float* seq_sum, int32_t* seq_cnt, int32_t* seq_nclip, int B, int64_t N,
                    void* stream) {
  if (B < 0 || N < 0 || N >= (1ll << 31)) return COPRIS_EINVAL;
  if (!(eps_low >= 0.0f) || !(eps_low < 1.0f) || !(eps_high >= 0.0f) || !(eps_high < INFINITY))
    return COPRIS_EINVAL;
  if (B == 0) return N == 0 ? COPRIS_OK : COPRIS_EINVAL;
  if (!cu_seqlens || !split || !seq_sum || !seq_cnt || !seq_nclip) return COPRIS_EINVAL;
  if (N > 0 && (!logp_cur || !logp_buf || !logp_roll || !ratio || !ratio_clipped))
    return COPRIS_EINVAL;
  if (!aligned16(logp_cur) || !aligned16(logp_buf) || !aligned16(logp_roll) || !aligned16(ratio) ||
      !aligned16(ratio_clipped) || (mask && !aligned16(mask)))
    return COPRIS_EINVAL;
  (void)hipGetLastError();
  return copris::launch_is_ratio(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, eps_low,
                          eps_high, ratio, ratio_clipped, seq_sum, seq_cnt, seq_nclip, B,
                          static_cast<hipStream_t>(stream));
}

int copris_grpo_surrogate(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                          const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                          const float* adv, float eps_low, float eps_high, float* surr, float* grad,
                          float* seq_surr, int32_t* seq_cnt, float* objective, int B, int64_t N,
                          void* stream) {
  if (B < 0 || N < 0 || N >= (1ll << 31)) return COPRIS_EINVAL;
  if (!(eps_low >= 0.0f) || !(eps_low < 1.0f) || !(eps_high >= 0.0f) || !(eps_high < INFINITY))
    return COPRIS_EINVAL;
  if (!objective) return COPRIS_EINVAL;
  if (B == 0 && N != 0) return COPRIS_EINVAL;
  if (B > 0 && (!cu_seqlens || !split || !adv || !seq_surr || !seq_cnt)) return COPRIS_EINVAL;
  if (N > 0 && (!logp_cur || !logp_buf || !logp_roll || !surr || !grad)) return COPRIS_EINVAL;
  if (!aligned16(logp_cur) || !aligned16(logp_buf) || !aligned16(logp_roll) || !aligned16(surr) ||
      !aligned16(grad) || (mask && !aligned16(mask)))
    return COPRIS_EINVAL;
  (void)hipGetLastError();
  return copris::launch_grpo_surrogate(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, adv,
                                       eps_low, eps_high, surr, grad, seq_surr, seq_cnt, objective, B,
                                       static_cast<hipStream_t>(stream));
}

}  // extern "C"
