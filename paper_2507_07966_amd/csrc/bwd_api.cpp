// prefix_attn_backward: argument checks on the host, then the launches (pre-pass, dQ pass,
// dK/dV pass over the prefix keys, dK/dV pass over the rollouts' own keys) on the caller's
// stream.  Nothing here allocates or synchronises (the timed variant waits for its events).
#include <hip/hip_runtime_api.h>

#include "bwd.h"

namespace {

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

struct BackwardArgs {
  const void *q, *k_prefix, *v_prefix, *k_suffix, *v_suffix, *out, *d_out, *lse;
  void *dq, *dk_prefix, *dv_prefix, *dk_suffix, *dv_suffix, *workspace;
  size_t workspace_bytes;
};

// When `ev` is non-null it holds 5 events recorded before, between and after the four stages.
int enqueue_backward(const prefix_attn_plan_t* plan, const BackwardArgs& x, void* hip_stream, hipEvent_t* ev) {
  if (!plan) return PA_ERR_NULL;
  const prefix_attn_desc_t& d = plan->desc;
  const bool has_prefix = d.prefix_len > 0;
  const void* always[] = {x.q, x.k_suffix, x.v_suffix, x.out, x.d_out, x.lse,
                          x.dq, x.dk_suffix, x.dv_suffix, x.workspace};
  for (const void* p : always) {
    if (!p) return PA_ERR_NULL;
  }
  const void* with_prefix[] = {x.k_prefix, x.v_prefix, x.dk_prefix, x.dv_prefix};
  if (has_prefix)
    for (const void* p : with_prefix) {
      if (!p) return PA_ERR_NULL;
    }
  for (const void* p : always) {
    if (misaligned(p)) return PA_ERR_ALIGN;
  }
  if (has_prefix)
    for (const void* p : with_prefix) {
      if (misaligned(p)) return PA_ERR_ALIGN;
    }
  if (x.workspace_bytes < plan->bws_bytes) return PA_ERR_WORKSPACE;
  // the dK/dV pass addresses a kv head's stacked rows with 32-bit byte offsets
  if (d.dtype == PA_BF16 && plan->Mpad * d.head_dim * 2 >= ((int64_t)1 << 31)) return PA_ERR_UNSUPPORTED;
  if (d.device < 0) return PA_ERR_UNSUPPORTED;  // host-only plan
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess || cur != d.device) return PA_ERR_HIP;  // the plan's device must be current

  hipStream_t hs = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(x.workspace);
  float* delta = reinterpret_cast<float*>(ws + plan->boff_delta);
  float* lse_th = reinterpret_cast<float*>(ws + plan->boff_lse_th);
  const bool bf16 = d.dtype == PA_BF16;

  // ---- stage 0: delta and (bf16) the streamed layouts, transposed K images
  if (ev && hipEventRecord(ev[0], hs) != hipSuccess) return PA_ERR_HIP;
  pa::BwdPrepArgs p{};
  p.q = x.q;
  p.out = x.out;
  p.d_out = x.d_out;
  p.lse = static_cast<const float*>(x.lse);
  p.delta = delta;
  p.lse_th = lse_th;
  p.T = plan->T;
  p.Mpad = plan->Mpad;
  p.Hq = d.num_q_heads;
  p.Hkv = d.num_kv_heads;
  p.D = d.head_dim;
  p.group = plan->group;
  p.dtype = d.dtype;
  if (bf16) {
    p.qs = ws + plan->boff_qs;
    p.dos = ws + plan->boff_dos;
    p.lse2s = reinterpret_cast<float*>(ws + plan->boff_lse2s);
    p.deltas = reinterpret_cast<float*>(ws + plan->boff_deltas);
    p.toks = reinterpret_cast<int32_t*>(ws + plan->boff_toks);
  }
  if (pa::launch_bwd_prep(p, hip_stream) != 0) return PA_ERR_HIP;
  if (bf16) {  // the same tile-image builder as for V in the forward, applied to K
    pa::VtArgs t{};
    t.v_prefix = x.k_prefix;
    t.v_suffix = x.k_suffix;
    t.vt_prefix = ws + plan->boff_ktp;
    t.vt_suffix = ws + plan->boff_kts;
    t.cu = plan->d_cu;
    t.vt_off = plan->d_vt_off;
    t.P = d.prefix_len;
    t.tiles_prefix = plan->tiles_prefix;
    t.tiles_suffix = plan->tiles_suffix;
    t.G = d.num_rollouts;
    t.Hkv = d.num_kv_heads;
    t.D = d.head_dim;
    t.order_32x32 = true;  // the dQ pass contracts with 32 x 32 x 16 MFMAs
    if (pa::launch_vt_images(t, hip_stream) != 0) return PA_ERR_HIP;
  }
  if (ev && hipEventRecord(ev[1], hs) != hipSuccess) return PA_ERR_HIP;

  if (!bf16) {
    pa::BwdF32Args f{};
    f.q = x.q;
    f.d_out = x.d_out;
    f.k_prefix = x.k_prefix;
    f.v_prefix = x.v_prefix;
    f.k_suffix = x.k_suffix;
    f.v_suffix = x.v_suffix;
    f.lse = lse_th;
    f.delta = delta;
    f.dq = x.dq;
    f.dk_prefix = x.dk_prefix;
    f.dv_prefix = x.dv_prefix;
    f.dk_suffix = x.dk_suffix;
    f.dv_suffix = x.dv_suffix;
    f.cu = plan->d_cu;
    f.T = plan->T;
    f.P = d.prefix_len;
    f.G = d.num_rollouts;
    f.Hq = d.num_q_heads;
    f.Hkv = d.num_kv_heads;
    f.D = d.head_dim;
    f.group = plan->group;
    f.scale = d.softmax_scale;
    if (pa::launch_bwd_dq_f32(f, hip_stream) != 0) return PA_ERR_HIP;
    if (ev && hipEventRecord(ev[2], hs) != hipSuccess) return PA_ERR_HIP;
    if (pa::launch_bwd_dkv_f32(f, hip_stream) != 0) return PA_ERR_HIP;
    if (ev && (hipEventRecord(ev[3], hs) != hipSuccess || hipEventRecord(ev[4], hs) != hipSuccess)) return PA_ERR_HIP;
    return PA_OK;
  }

  // ---- stage 1: dQ
  pa::BwdDqArgs a{};
  a.q = x.q;
  a.d_out = x.d_out;
  a.k_prefix = x.k_prefix;
  a.v_prefix = x.v_prefix;
  a.k_suffix = x.k_suffix;
  a.v_suffix = x.v_suffix;
  a.kt_prefix = ws + plan->boff_ktp;
  a.kt_suffix = ws + plan->boff_kts;
  a.lse2s = reinterpret_cast<const float*>(ws + plan->boff_lse2s);
  a.deltas = reinterpret_cast<const float*>(ws + plan->boff_deltas);
  a.Mpad = plan->Mpad;
  a.dq = x.dq;
  a.dq_partial = reinterpret_cast<float*>(ws + plan->boff_dqpart);
  a.key_splits = plan->key_splits;
  a.T = plan->T;
  a.items = plan->d_dq_items;
  a.num_items = (int64_t)plan->dq_items.size();
  a.cu = plan->d_cu;
  a.vt_off = plan->d_vt_off;
  a.P = d.prefix_len;
  a.tiles_prefix = plan->tiles_prefix;
  a.tiles_suffix = plan->tiles_suffix;
  a.Hq = d.num_q_heads;
  a.Hkv = d.num_kv_heads;
  a.D = d.head_dim;
  a.group = plan->group;
  a.scale = d.softmax_scale;
  if (pa::launch_bwd_dq_bf16(a, hip_stream) != 0) return PA_ERR_HIP;
  if (ev && hipEventRecord(ev[2], hs) != hipSuccess) return PA_ERR_HIP;

  // ---- stages 2, 3: dK/dV of the prefix keys, then of the rollouts' own keys
  pa::BwdDkvArgs kv{};
  kv.qs = ws + plan->boff_qs;
  kv.dos = ws + plan->boff_dos;
  kv.lse2s = reinterpret_cast<const float*>(ws + plan->boff_lse2s);
  kv.deltas = reinterpret_cast<const float*>(ws + plan->boff_deltas);
  kv.toks = reinterpret_cast<const int32_t*>(ws + plan->boff_toks);
  kv.cu = plan->d_cu;
  kv.T = plan->T;
  kv.Mpad = plan->Mpad;
  kv.Hkv = d.num_kv_heads;
  kv.D = d.head_dim;
  kv.group = plan->group;
  kv.scale = d.softmax_scale;
  kv.partial = reinterpret_cast<float*>(ws + plan->boff_part);
  if (has_prefix) {
    kv.k = x.k_prefix;
    kv.v = x.v_prefix;
    kv.dk = x.dk_prefix;
    kv.dv = x.dv_prefix;
    kv.P = d.prefix_len;
    kv.items = plan->d_key_items[0];
    kv.num_items = (int64_t)plan->key_items[0].size();
    kv.causal = false;
    kv.partials = kv.reduce = plan->row_splits > 1;
    kv.splits = plan->row_splits;
    if (pa::launch_bwd_dkv_bf16(kv, hip_stream) != 0) return PA_ERR_HIP;
  }
  if (ev && hipEventRecord(ev[3], hs) != hipSuccess) return PA_ERR_HIP;
  // the rollouts' own keys: the masked kernel (on the tiles that need the mask only, when the plan splits the
  // pass), then the mask-free kernel on the other tiles and the sum of the two partial gradients
  kv.k = x.k_suffix;
  kv.v = x.v_suffix;
  kv.dk = x.dk_suffix;
  kv.dv = x.dv_suffix;
  kv.P = plan->T;
  kv.items = plan->d_key_items[1];
  kv.num_items = (int64_t)plan->key_items[1].size();
  kv.causal = true;
  kv.partials = plan->suffix_split;
  kv.reduce = false;
  kv.splits = 2;
  if (pa::launch_bwd_dkv_bf16(kv, hip_stream) != 0) return PA_ERR_HIP;
  if (plan->suffix_split) {
    kv.items = plan->d_key_items_full;
    kv.num_items = (int64_t)plan->key_items_full.size();
    kv.causal = false;
    kv.reduce = true;
    if (pa::launch_bwd_dkv_bf16(kv, hip_stream) != 0) return PA_ERR_HIP;
  }
  if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return PA_ERR_HIP;
  return PA_OK;
}

}  // namespace

extern "C" {

int prefix_attn_backward(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix, const void* v_prefix,
                         const void* k_suffix, const void* v_suffix, const void* out, const void* d_out,
                         const float* lse, void* dq, void* dk_prefix, void* dv_prefix, void* dk_suffix,
                         void* dv_suffix, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const BackwardArgs x{q,  k_prefix,  v_prefix,  k_suffix,  v_suffix,  out,       d_out,          lse,
                       dq, dk_prefix, dv_prefix, dk_suffix, dv_suffix, workspace, workspace_bytes};
  return enqueue_backward(plan, x, hip_stream, nullptr);
}

int prefix_attn_backward_timed(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_suffix, const void* v_suffix, const void* out,
                               const void* d_out, const float* lse, void* dq, void* dk_prefix,
                               void* dv_prefix, void* dk_suffix, void* dv_suffix, void* workspace,
                               size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
  if (!plan || !kernel_ms) return PA_ERR_NULL;
  if (plan->desc.device < 0) return PA_ERR_UNSUPPORTED;  // host-only plan: no events either
  const BackwardArgs x{q,  k_prefix,  v_prefix,  k_suffix,  v_suffix,  out,       d_out,          lse,
                       dq, dk_prefix, dv_prefix, dk_suffix, dv_suffix, workspace, workspace_bytes};
  hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
  int st = PA_OK;
  for (int i = 0; i < 5 && st == PA_OK; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) st = PA_ERR_HIP;
  if (st == PA_OK) st = enqueue_backward(plan, x, hip_stream, ev);
  if (st == PA_OK && hipEventSynchronize(ev[4]) != hipSuccess) st = PA_ERR_HIP;
  for (int i = 0; i < 4 && st == PA_OK; ++i)
    if (hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = PA_ERR_HIP;
  for (int i = 0; i < 5; ++i)
    if (ev[i]) (void)hipEventDestroy(ev[i]);
  return st;
}

}  // extern "C"
