// prefix_attn_forward / prefix_attn_lse: argument checks on the host, then the launches
// (prefix pass, suffix pass, and a merge where the suffix pass does not do it) on the caller's stream.  Nothing here allocates or
// synchronises.
#include <hip/hip_runtime.h>

#include <mutex>

#include "common.h"

// Workspace of prefix_attn_forward_static: one array per GPU, part of the library's device image, so that
// entry point never has to ask anyone for memory.  In host code this name is only a handle for
// hipGetSymbolAddress; the array's memory is reached through the pointer static_scratch() returns.
static __device__ __align__(256) unsigned char scratch[PA_STATIC_SCRATCH_BYTES];

namespace pa {

// Device address of `scratch` on `device`, which must be the current device.  Looked up once per device
// and kept (every GPU holds its own copy of the array at its own address).
int static_scratch(int device, void** ptr_out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex lock;
  static void* ptrs[MAX_DEVICES] = {};
  if (device < 0 || device >= MAX_DEVICES) return PA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(lock);
  if (!ptrs[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return PA_ERR_HIP;
    }
    ptrs[device] = p;
  }
  *ptr_out = ptrs[device];
  return PA_OK;
}

}  // namespace pa

namespace {

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// What a forward call leaves behind.
enum Mode {
  FULL = 0,            // out in the plan's dtype, merged LSE in the workspace
  PARTIAL_ALL = 1,     // fp32 partial over prefix shard + suffix keys, in caller buffers
  PARTIAL_PREFIX = 2,  // fp32 partial over the prefix shard only, in caller buffers
};

// Checks, then the launches (layout pre-pass, prefix pass, suffix pass, merge).  When `ev` is
// non-null it holds 5 events recorded before, between and after them.  In the partial modes
// `out` is the fp32 partial output and `lse_partial` its [T, Hq] LSE.
int enqueue_forward(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix, const void* v_prefix,
                    const void* k_suffix, const void* v_suffix, void* out, void* workspace, size_t workspace_bytes,
                    void* hip_stream, hipEvent_t* ev, Mode mode = FULL, float* lse_partial = nullptr) {
  if (!plan || !q || !out || !workspace) return PA_ERR_NULL;
  const bool with_suffix = mode != PARTIAL_PREFIX;
  if (with_suffix && (!k_suffix || !v_suffix)) return PA_ERR_NULL;
  if (mode != FULL && !lse_partial) return PA_ERR_NULL;
  const prefix_attn_desc_t& d = plan->desc;
  const bool has_prefix = d.prefix_len > 0;
  if (!with_suffix && !has_prefix) return PA_ERR_SHAPE;  // a prefix-only partial over no keys
  if (has_prefix && (!k_prefix || !v_prefix)) return PA_ERR_NULL;
  if (misaligned(q) || misaligned(out) || misaligned(workspace) || misaligned(lse_partial)) return PA_ERR_ALIGN;
  if (with_suffix && (misaligned(k_suffix) || misaligned(v_suffix))) return PA_ERR_ALIGN;
  if (has_prefix && (misaligned(k_prefix) || misaligned(v_prefix))) return PA_ERR_ALIGN;
  if (workspace_bytes < plan->ws_bytes) return PA_ERR_WORKSPACE;
  if (d.device < 0) return PA_ERR_UNSUPPORTED;  // host-only plan
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess || cur != d.device) return PA_ERR_HIP;  // the plan's device must be current

  char* ws = static_cast<char*>(workspace);
  float* o1 = reinterpret_cast<float*>(ws + plan->off_o1);
  float* o2 = reinterpret_cast<float*>(ws + plan->off_o2);
  float* lse1 = reinterpret_cast<float*>(ws + plan->off_lse1);
  float* lse2 = reinterpret_cast<float*>(ws + plan->off_lse2);
  float* lse = reinterpret_cast<float*>(ws + plan->off_lse);

  pa::PassArgs a{};
  a.q = q;
  a.cu = plan->d_cu;
  a.Hq = d.num_q_heads;
  a.Hkv = d.num_kv_heads;
  a.D = d.head_dim;
  a.group = plan->group;
  a.scale = d.softmax_scale;
  a.part_rows = plan->T * d.num_q_heads;
  a.flags = reinterpret_cast<int32_t*>(ws + plan->off_flags);  // bf16 passes only
  // With key splits the prefix pass leaves `ks` partials in the workspace and an n-way merge
  // combines them (and the suffix partial) instead of the two-way merge.
  const int ks = plan->key_splits;
  auto merge_splits = [&](bool suffix_too, void* dst, int32_t dst_dtype, float* lse_th) {
    pa::MergeNArgs m{};
    for (int i = 0; i < ks; ++i) {
      m.o[i] = o1 + (size_t)i * a.part_rows * d.head_dim;
      m.lse[i] = lse1 + (size_t)i * a.part_rows;
    }
    if (suffix_too) {
      m.o[ks] = o2;
      m.lse[ks] = lse2;
    }
    m.out = dst;
    m.lse_th_out = lse_th;
    m.T = plan->T;
    m.n = ks + (suffix_too ? 1 : 0);
    m.Hq = d.num_q_heads;
    m.D = d.head_dim;
    m.dtype = dst_dtype;
    return pa::launch_merge_n(m, hip_stream);
  };
  auto launch_pass = (d.dtype == PA_BF16) ? pa::launch_pass_bf16 : pa::launch_pass_f32;

  hipStream_t hs = static_cast<hipStream_t>(hip_stream);
  if (ev && hipEventRecord(ev[0], hs) != hipSuccess) return PA_ERR_HIP;
  if (d.dtype == PA_BF16) {  // layout pre-pass: V^T tile images for the MFMA passes
    pa::VtArgs t{};
    t.v_prefix = v_prefix;
    t.v_suffix = v_suffix;
    t.vt_prefix = ws + plan->off_vtp;
    t.vt_suffix = ws + plan->off_vts;
    t.cu = plan->d_cu;
    t.vt_off = plan->d_vt_off;
    t.P = d.prefix_len;
    t.tiles_prefix = plan->tiles_prefix;
    t.tiles_suffix = with_suffix ? plan->tiles_suffix : 0;
    t.G = d.num_rollouts;
    t.Hkv = d.num_kv_heads;
    t.D = d.head_dim;
    t.order_32x32 = false;  // the attention passes contract with 16 x 16 x 32 MFMAs
    if (pa::launch_vt_images(t, hip_stream) != 0) return PA_ERR_HIP;
  }
  if (ev && hipEventRecord(ev[1], hs) != hipSuccess) return PA_ERR_HIP;
  // bf16, unsplit short prefix (the plan decides), own keys included: one sweep over [prefix | own keys] per
  // block of rows does the work of the prefix pass, the suffix pass and the merge (the sweep list carries both
  // extents); it leaves the result of the call, or the fp32 partial of a shard that also holds the own keys
  const bool sweep = with_suffix && !plan->sweep_items.empty();
  if (has_prefix && !sweep) {
    a.k = k_prefix;
    a.v = v_prefix;
    a.vt = ws + plan->off_vtp;
    a.vt_off = nullptr;
    a.vt_tiles_per_head = plan->tiles_prefix;
    const bool direct = !with_suffix && ks == 1;  // an unsplit prefix-only partial goes straight to the caller
    a.o_part = direct ? static_cast<float*>(out) : o1;
    a.lse_part = direct ? lse_partial : lse1;
    a.items = plan->d_items[0];
    a.num_items = (int64_t)plan->items[0].size();
    a.causal = false;
    if (launch_pass(a, hip_stream) != 0) return PA_ERR_HIP;
  }
  if (ev && hipEventRecord(ev[2], hs) != hipSuccess) return PA_ERR_HIP;
  if (!with_suffix) {
    if (ks > 1 && merge_splits(false, out, PA_F32, lse_partial) != 0) return PA_ERR_HIP;
    return PA_OK;
  }
  a.k = k_suffix;
  a.v = v_suffix;
  a.vt = ws + plan->off_vts;
  a.vt_off = plan->d_vt_off;
  a.vt_tiles_per_head = plan->tiles_suffix;
  a.o_part = o2;
  a.lse_part = lse2;
  a.items = plan->d_items[1];
  a.num_items = (int64_t)plan->items[1].size();
  a.causal = true;
  // bf16, whole call, unsplit prefix: the suffix pass combines its result with the prefix partial in its
  // epilogue and writes `out` and the merged LSE itself (no merge launch, no suffix partial in memory)
  const bool fused = mode == FULL && d.dtype == PA_BF16 && ks == 1;
  if (fused) {
    a.epilogue = (has_prefix && !sweep) ? 2 : 1;
    a.o1 = o1;
    a.lse1 = lse1;
    a.out_final = out;
    a.lse_final = lse;
  }
  if (sweep) {
    a.sweep_prefix = true;
    a.k_pre = k_prefix;
    a.vt_pre = ws + plan->off_vtp;
    a.vt_pre_tiles_per_head = plan->tiles_prefix;
    a.items = plan->d_sweep_items;
    a.num_items = (int64_t)plan->sweep_items.size();
    if (!fused) {  // a shard's partial: straight into the caller's buffers
      a.o_part = static_cast<float*>(out);
      a.lse_part = lse_partial;
    }
  }
  if (launch_pass(a, hip_stream) != 0) return PA_ERR_HIP;

  if (ev && hipEventRecord(ev[3], hs) != hipSuccess) return PA_ERR_HIP;
  if (fused || sweep) {
    if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return PA_ERR_HIP;
    return PA_OK;
  }
  if (ks > 1) {
    if (merge_splits(true, out, mode == FULL ? d.dtype : (int32_t)PA_F32, mode == FULL ? lse : lse_partial) != 0)
      return PA_ERR_HIP;
    if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return PA_ERR_HIP;
    return PA_OK;
  }
  pa::MergeArgs m{};
  m.o1 = o1;
  m.lse1 = lse1;
  m.o2 = o2;
  m.lse2 = lse2;
  m.out = out;
  m.lse = mode == FULL ? lse : lse_partial;
  m.rows = plan->T * d.num_q_heads;
  m.D = d.head_dim;
  m.dtype = mode == FULL ? d.dtype : (int32_t)PA_F32;
  m.has_prefix = has_prefix;
  if (pa::launch_merge(m, hip_stream) != 0) return PA_ERR_HIP;
  if (ev && hipEventRecord(ev[4], hs) != hipSuccess) return PA_ERR_HIP;
  return PA_OK;
}

}  // namespace

extern "C" {

int prefix_attn_forward(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix, const void* v_prefix,
                        const void* k_suffix, const void* v_suffix, void* out, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  return enqueue_forward(plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, workspace, workspace_bytes, hip_stream,
                         nullptr);
}

int prefix_attn_forward_static(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                               const void* v_prefix, const void* k_suffix, const void* v_suffix, void* out,
                               float* lse_out, void* hip_stream) {
  if (!plan) return PA_ERR_NULL;
  if (plan->ws_bytes > (size_t)PA_STATIC_SCRATCH_BYTES) return PA_ERR_WORKSPACE;
  if (plan->desc.device < 0) return PA_ERR_UNSUPPORTED;  // host-only plan
  if (reinterpret_cast<uintptr_t>(lse_out) & 15u) return PA_ERR_ALIGN;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess || cur != plan->desc.device) return PA_ERR_HIP;
  void* ws = nullptr;
  int st = pa::static_scratch(cur, &ws);  // already resolved when the plan was made; a table look-up here
  if (st != PA_OK) return st;
  st = enqueue_forward(plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, ws, PA_STATIC_SCRATCH_BYTES, hip_stream,
                       nullptr);
  if (st != PA_OK || !lse_out) return st;
  return prefix_attn_lse(plan, ws, lse_out, hip_stream);
}

int prefix_attn_forward_timed(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                              const void* v_prefix, const void* k_suffix, const void* v_suffix, void* out,
                              void* workspace, size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
  if (!plan || !kernel_ms) return PA_ERR_NULL;
  if (plan->desc.device < 0) return PA_ERR_UNSUPPORTED;  // host-only plan: no events either
  hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
  int st = PA_OK;
  for (int i = 0; i < 5 && st == PA_OK; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) st = PA_ERR_HIP;
  if (st == PA_OK)
    st = enqueue_forward(plan, q, k_prefix, v_prefix, k_suffix, v_suffix, out, workspace, workspace_bytes, hip_stream, ev);
  if (st == PA_OK && hipEventSynchronize(ev[4]) != hipSuccess) st = PA_ERR_HIP;
  for (int i = 0; i < 4 && st == PA_OK; ++i)
    if (hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = PA_ERR_HIP;
  for (int i = 0; i < 5; ++i)
    if (ev[i]) (void)hipEventDestroy(ev[i]);
  return st;
}

int prefix_attn_forward_partial(const prefix_attn_plan_t* plan, const void* q, const void* k_prefix,
                                const void* v_prefix, const void* k_suffix, const void* v_suffix,
                                int32_t include_suffix, float* o_partial, float* lse_partial, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  return enqueue_forward(plan, q, k_prefix, v_prefix, k_suffix, v_suffix, o_partial, workspace, workspace_bytes,
                         hip_stream, nullptr, include_suffix ? PARTIAL_ALL : PARTIAL_PREFIX, lse_partial);
}

int prefix_attn_merge_partials(const prefix_attn_plan_t* plan, int32_t n, const float* const* o_partials,
                               const float* const* lse_partials, void* out, float* lse_out, void* hip_stream) {
  if (!plan || !o_partials || !lse_partials || !out) return PA_ERR_NULL;
  if (n < 1 || n > PA_MAX_PARTIALS) return PA_ERR_SHAPE;
  pa::MergeNArgs a{};
  for (int i = 0; i < n; ++i) {
    if (!o_partials[i] || !lse_partials[i]) return PA_ERR_NULL;
    if (misaligned(o_partials[i]) || misaligned(lse_partials[i])) return PA_ERR_ALIGN;
    a.o[i] = o_partials[i];
    a.lse[i] = lse_partials[i];
  }
  if (misaligned(out) || misaligned(lse_out)) return PA_ERR_ALIGN;
  if (plan->desc.device < 0) return PA_ERR_UNSUPPORTED;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess || cur != plan->desc.device) return PA_ERR_HIP;
  a.out = out;
  a.lse_out = lse_out;
  a.T = plan->T;
  a.n = n;
  a.Hq = plan->desc.num_q_heads;
  a.D = plan->desc.head_dim;
  a.dtype = plan->desc.dtype;
  if (pa::launch_merge_n(a, hip_stream) != 0) return PA_ERR_HIP;
  return PA_OK;
}

int prefix_attn_lse(const prefix_attn_plan_t* plan, const void* workspace, float* lse_out, void* hip_stream) {
  if (!plan || !workspace || !lse_out) return PA_ERR_NULL;
  if (misaligned(workspace) || misaligned(lse_out)) return PA_ERR_ALIGN;
  if (plan->desc.device < 0) return PA_ERR_UNSUPPORTED;
  const float* lse = reinterpret_cast<const float*>(static_cast<const char*>(workspace) + plan->off_lse);
  if (pa::launch_lse_export(lse, lse_out, plan->T, plan->desc.num_q_heads, hip_stream) != 0) return PA_ERR_HIP;
  return PA_OK;
}

}  // extern "C"
