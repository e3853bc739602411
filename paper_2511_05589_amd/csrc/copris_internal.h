// Host-side declarations shared by the C ABI and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace copris {

// Checks hipGetLastError() after a launch; on failure records "<kernel>: <hip error>" for
// copris_last_error_detail() and returns false.
bool launch_ok(const char* kernel_name);
// Records "<what>: <hip error>" for copris_last_error_detail().
void set_error_detail(const char* what, hipError_t e);
// Calls the profiling hook (if one is set) before (phase 0) / after (phase 1) a launch.
void launch_hook(const char* kernel_name, int phase, hipStream_t stream);
constexpr int kErrLaunch = -4;   // COPRIS_ELAUNCH

// Around every kernel launch of a launcher whose stream variable is called `stream`.
#define COPRIS_PRE(name) ::copris::launch_hook(name, 0, stream)
#define COPRIS_POST(name)                                          \
  do {                                                             \
    if (!::copris::launch_ok(name)) return ::copris::kErrLaunch;   \
    ::copris::launch_hook(name, 1, stream);                        \
  } while (0)

// ---- decode attention -------------------------------------------------------
constexpr int kAttnChunkTokens = 512;   // split-K granularity along the context
constexpr int kAttnMaxGroup = 16;       // query heads per kv head, at most
constexpr int kAttnWaves = 256 * 8;     // persistent wavefronts of the tuned split kernel (8 per CU)

// Workspace carve-up (byte offsets from a 256-byte aligned base).
struct AttnWorkspace {
  size_t hdr;       // int32[64]:  [0] number of (seq, chunk) entries, [1] work counter
  size_t seq_off;   // int32[C+1]: first list entry (generic path) / page prefix (tuned path) of every sequence
  size_t list;      // int2[]: (seq, chunk) items (generic path) / int4 start cursor per wavefront (tuned path)
  size_t ml;        // float2[max_list*Hkv*g]: running max (log2 domain) and sum of weights
  size_t acc;       // float[max_list*Hkv*g*D]: un-normalised weighted value sums
  size_t total;
  int64_t max_list;
};
AttnWorkspace attn_workspace_layout(int C, int Hq, int Hkv, int D, int page_size, int max_pages);

int launch_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_len, void* out, float* lse,
                       void* workspace, int C, int Hq, int Hkv, int D, int page_size,
                       int max_pages, float scale, int dtype, hipStream_t stream);

// ---- re-prefill attention ----------------------------------------------------
bool prefill_attn_supported(int Hq, int Hkv, int D, int page_size, int dtype);
int launch_prefill_attn(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                        const int32_t* block_table, void* k_cache, void* v_cache, void* out,
                        float* lse, int B, int Hq, int Hkv, int max_pages, int max_seqlen,
                        float scale, hipStream_t stream);

// ---- LM head ----------------------------------------------------------------
struct LmWorkspace {
  size_t part;      // LmPartial[C * n_tiles]
  size_t total;
  int n_tiles;
};
LmWorkspace lm_workspace_layout(int C, int H, int V);

size_t lm_token_workspace_bytes(int M, int H, int V, int dtype);
int launch_lmhead_token_logprob(const void* hidden, const void* weight, const int32_t* tokens,
                                float temperature, float* logprob, float* lse, void* workspace,
                                int M, int H, int V, int dtype, hipStream_t stream);

int launch_lmhead_logprob(const void* hidden, const void* weight, const int64_t* seq_id,
                          const int32_t* step, uint64_t seed, float temperature, int32_t* token,
                          float* logprob, float* lse, void* workspace, int C, int H, int V,
                          int dtype, hipStream_t stream);

// the sampling call with its partials in the library's own static device array
size_t lm_noalloc_scratch_limit();
size_t lm_noalloc_scratch_needed(int C, int H, int V, int dtype);
int launch_lmhead_logprob_noalloc(const void* hidden, const void* weight, const int64_t* seq_id,
                                  const int32_t* step, uint64_t seed, float temperature,
                                  int32_t* token, float* logprob, float* lse, int C, int H, int V,
                                  int dtype, hipStream_t stream);

// ---- IS ratio ---------------------------------------------------------------
int launch_is_ratio(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                    const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                    float eps_low, float eps_high, float* ratio, float* ratio_clipped,
                    float* seq_sum, int32_t* seq_cnt, int32_t* seq_nclip, int B,
                    hipStream_t stream);
int launch_grpo_surrogate(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                          const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                          const float* adv, float eps_low, float eps_high, float* surr, float* grad,
                          float* seq_surr, int32_t* seq_cnt, float* objective, int B,
                          hipStream_t stream);

}  // namespace copris
