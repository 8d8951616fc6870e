// Internal declarations of the response-token log-probability kernels.
#pragma once

#include <cstdint>

namespace pa {

constexpr int LP_TILE = 256;  // vocabulary rows and tokens per workgroup tile

struct LogprobArgs {
  const void* hidden;      // [N, d] bf16
  const void* lm_head;     // [V, d] bf16
  const int32_t* targets;  // [N]
  float* logprob;          // [N]
  float* lse;              // [N] or null
  float* partials;         // workspace: [ceil(V / LP_TILE)][N] pairs (m, l)
  float* target_logit;     // workspace: [N]
  int64_t N;
  int32_t d, V;
  float logit_scale;
};
int launch_logprob(const LogprobArgs& a, void* stream);
int launch_group_advantages(const float* rewards, float* adv, int G, int num_groups, void* stream);

}  // namespace pa
