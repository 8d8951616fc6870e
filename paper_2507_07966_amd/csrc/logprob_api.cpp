// token_logprob_* and grpo_group_advantages: argument checks on the host, then the launches on
// the caller's stream.  Nothing here allocates or synchronises.
#include <hip/hip_runtime_api.h>

#include <cmath>

#include "logprob.h"
#include "prefix_attn.h"

namespace {

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(int64_t N, int32_t d, int32_t V) {
  if (N < 1 || d < 1 || V < 1) return PA_ERR_SHAPE;
  if (N > ((int64_t)1 << 31) - 1) return PA_ERR_SHAPE;
  if (d % 64 != 0) return PA_ERR_UNSUPPORTED;  // the kernel steps over the hidden dimension 64 channels at a time
  return PA_OK;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
size_t partial_bytes(int64_t N, int32_t V) {
  const size_t blocks = (size_t)((V + pa::LP_TILE - 1) / pa::LP_TILE);
  return align_up(blocks * (size_t)N * 2 * sizeof(float), 256);
}

}  // namespace

extern "C" {

int token_logprob_workspace(int64_t num_tokens, int32_t hidden_dim, int32_t vocab, size_t* workspace_bytes_out) {
  if (!workspace_bytes_out) return PA_ERR_NULL;
  const int st = check_shape(num_tokens, hidden_dim, vocab);
  if (st != PA_OK) return st;
  *workspace_bytes_out = partial_bytes(num_tokens, vocab) + align_up((size_t)num_tokens * sizeof(float), 256);
  return PA_OK;
}

int token_logprob_forward(const void* hidden, const void* lm_head, const int32_t* targets, int64_t num_tokens,
                          int32_t hidden_dim, int32_t vocab, float logit_scale, float* logprob_out, float* lse_out,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!hidden || !lm_head || !targets || !logprob_out || !workspace) return PA_ERR_NULL;
  const int st = check_shape(num_tokens, hidden_dim, vocab);
  if (st != PA_OK) return st;
  if (!(logit_scale > 0.0f) || !std::isfinite(logit_scale)) return PA_ERR_SHAPE;
  if (misaligned(hidden) || misaligned(lm_head) || misaligned(targets) || misaligned(logprob_out) ||
      misaligned(lse_out) || misaligned(workspace))
    return PA_ERR_ALIGN;
  size_t need = 0;
  (void)token_logprob_workspace(num_tokens, hidden_dim, vocab, &need);
  if (workspace_bytes < need) return PA_ERR_WORKSPACE;
  pa::LogprobArgs a{};
  a.hidden = hidden;
  a.lm_head = lm_head;
  a.targets = targets;
  a.logprob = logprob_out;
  a.lse = lse_out;
  a.partials = static_cast<float*>(workspace);
  a.target_logit = reinterpret_cast<float*>(static_cast<char*>(workspace) + partial_bytes(num_tokens, vocab));
  a.N = num_tokens;
  a.d = hidden_dim;
  a.V = vocab;
  a.logit_scale = logit_scale;
  if (pa::launch_logprob(a, hip_stream) != 0) return PA_ERR_HIP;
  return PA_OK;
}

int grpo_group_advantages(const float* rewards, int32_t group_size, int32_t num_groups, float* advantages_out,
                          void* hip_stream) {
  if (!rewards || !advantages_out) return PA_ERR_NULL;
  if (group_size < 1 || num_groups < 0) return PA_ERR_SHAPE;
  if (pa::launch_group_advantages(rewards, advantages_out, group_size, num_groups, hip_stream) != 0) return PA_ERR_HIP;
  return PA_OK;
}

}  // extern "C"
