// Internal declarations of the backward pass (host side and kernel launchers).
//
// Given dO, the backward produces dQ, and dK/dV of the shared prefix and of every rollout's own
// tokens.  With W the softmax weights of a query row (recomputed from the saved LSE):
//   delta = <dO, O>,  dW_j = <dO, v_j>,  dS_j = W_j (dW_j - delta),
//   dQ = scale sum_j dS_j k_j,   dK_j = scale sum_rows dS_j q,   dV_j = sum_rows W_j dO.
// A prefix key/value sums over the rows of ALL rollouts and the q heads of its GQA group,
// because every rollout attends to the same cached video prefix (paper Sec. 5.1); the policy
// model is trained through this attention (Eq. 1, Sec. 5.2).
#pragma once

#include "common.h"

namespace pa {

struct BwdPrepArgs {
  const void* q;       // [T, Hq, D]
  const void* out;     // [T, Hq, D]
  const void* d_out;   // [T, Hq, D]
  const float* lse;    // [Hq, T] natural log, as exported after the forward
  float* delta;        // [T, Hq] out: <dO, O>            (fp32 path)
  float* lse_th;       // [T, Hq] out: LSE re-ordered     (fp32 path)
  // bf16 path only: per kv head, the stacked rows gathered into contiguous order
  void* qs;            // [Hkv][Mpad][D]
  void* dos;           // [Hkv][Mpad][D]
  float* lse2s;        // [Hkv][Mpad]  LSE * log2(e); rows past the end hold a huge value
  float* deltas;       // [Hkv][Mpad]  -<dO, O> per stacked row (negated)
  int32_t* toks;       // [Hkv][Mpad]  packed token index of the stacked row; INT32_MAX past the end
  int64_t T;
  int64_t Mpad;        // stacked rows per kv head rounded up to ROWS_PER_ROW_TILE
  int32_t Hq, Hkv, D, group, dtype;
};
int launch_bwd_prep(const BwdPrepArgs& a, void* stream);

struct BwdDqArgs {
  const void* q;         // [T, Hq, D]
  const void* d_out;     // [T, Hq, D]
  const void* k_prefix;  // [P, Hkv, D]
  const void* v_prefix;
  const void* k_suffix;  // [T, Hkv, D]
  const void* v_suffix;
  const void* kt_prefix;  // bf16: transposed K tile images [Hkv][tiles_prefix][D][64]
  const void* kt_suffix;  // bf16: [Hkv][tiles_suffix][D][64]
  const float* lse2s;     // [Hkv][Mpad] LSE * log2(e) per stacked row (from the pre-pass)
  const float* deltas;    // [Hkv][Mpad] -delta per stacked row
  void* dq;               // [T, Hq, D]
  float* dq_partial;      // key_splits > 1: fp32 partial dQ [key_splits][T][Hq][D]
  int32_t key_splits;
  int64_t T;
  const WorkItem* items;  // the plan's dQ list: (g, row0, c, causal extent, prefix key range, split)
  const int32_t* cu;
  const int32_t* vt_off;
  int64_t num_items, P, Mpad;
  int32_t tiles_prefix, tiles_suffix, Hq, Hkv, D, group;
  float scale;
};
int launch_bwd_dq_bf16(const BwdDqArgs& a, void* stream);

struct BwdDkvArgs {
  const void* k;        // prefix: [P, Hkv, D]; suffix: [T, Hkv, D]
  const void* v;
  const void* qs;       // stacked-row copies / images / statistics from the pre-pass
  const void* dos;
  const float* lse2s;
  const float* deltas;
  const int32_t* toks;
  void* dk;             // same shape as k
  void* dv;
  float* partial;       // partials == true: unscaled fp32 partial gradients [2][splits][P][Hkv][D]
  const KeyItem* items;
  const int32_t* cu;
  int64_t num_items, T, Mpad;
  int64_t P;            // keys (rows) of k / v / dk / dv: the prefix length, or T for the rollouts' own keys
  int32_t splits;       // partial-gradient slots (an item writes slot KeyItem::split)
  int32_t Hkv, D, group;
  float scale;
  bool causal;          // true: the masked kernel (keys indexed inside their rollout, rows from the key on);
                        // false: the mask-free kernel (keys indexed over the whole array, every streamed row sees them)
  bool partials;        // items leave fp32 partials instead of writing dk / dv
  bool reduce;          // after the launch, add the slots of `partial` into dk / dv (scaled, in the tensors' dtype)
};
int launch_bwd_dkv_bf16(const BwdDkvArgs& a, void* stream);

// fp32 path: plain kernels (one wavefront per query row / per key)
struct BwdF32Args {
  const void* q;
  const void* d_out;
  const void* k_prefix;
  const void* v_prefix;
  const void* k_suffix;
  const void* v_suffix;
  const float* lse;     // [T, Hq]
  const float* delta;   // [T, Hq]
  void* dq;
  void* dk_prefix;
  void* dv_prefix;
  void* dk_suffix;
  void* dv_suffix;
  const int32_t* cu;
  int64_t T, P;
  int32_t G, Hq, Hkv, D, group;
  float scale;
};
int launch_bwd_dq_f32(const BwdF32Args& a, void* stream);
int launch_bwd_dkv_f32(const BwdF32Args& a, void* stream);

}  // namespace pa
