// Internal declarations shared by the host side (plan, API) and the kernel launchers.
// Nothing here is part of the public C ABI (see include/prefix_attn.h).
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "prefix_attn.h"

namespace pa {

// Tile geometry of the two attention passes: one work item = ROWS_PER_ITEM stacked query
// rows of one (kv head, rollout); keys are swept in LDS tiles of KEYS_PER_TILE.
constexpr int ROWS_PER_ITEM = 256;
constexpr int WAVES_PER_ITEM = 8;   // wavefronts of the bf16 attention kernels' workgroup (32 rows each)
constexpr int KEYS_PER_TILE = 64;
// The layout the work lists are tuned for (MI355X): 256 compute units in 8 XCDs, workgroup n dispatched to
// XCD n % 8.  A plan for a device that reports another compute-unit count (a partitioned GPU, say) uses that
// count and does not interleave its lists over XCDs; host-only plans assume this layout.
constexpr int NUM_XCD = 8;
constexpr int NUM_CU = 256;
// Whole bf16 calls with at most this many prefix tiles (65,536 keys) run as one sweep over [prefix | own keys]
// per block of rows: no partial results, no second launch.  Longer prefixes keep the separate prefix and suffix
// passes: there the equally long items of the prefix pass, which walk the prefix in step and share its tiles
// in L2, outweigh the suffix pass they cost (measured: the sweep is 0.8 % faster at 512 prefix tiles, 0.7 %
// slower at 3,600; break-even near 1,000).
constexpr int SWEEP_MAX_PREFIX_TILES = 1024;

// One entry of a pass's work list.  g < 0 marks a padding entry (the workgroup exits).
struct WorkItem {
  int32_t g;      // rollout
  int32_t row0;   // first stacked row inside the rollout, m = i * group + (h % group)
  int32_t c;      // kv head
  int32_t nkeys;  // keys swept: the item's share of P in the prefix pass, causal extent in the suffix pass
  int32_t key0;   // prefix pass: first prefix key swept (a multiple of KEYS_PER_TILE); suffix pass: 0
  int32_t split;  // prefix pass: which key split this is (its partial lands in slot `split`); else 0
  int32_t pkeys;  // backward dQ list only: prefix keys [key0, key0 + pkeys) swept before the nkeys own keys
  int32_t pad_;
};

// Backward tile geometry.  The key-stationary pass (dK/dV) gives a workgroup KEYS_PER_KEY_ITEM
// keys of one kv head and streams stacked query rows past them in tiles of ROWS_PER_ROW_TILE.
// Stacked rows of kv head c are numbered over all packed tokens: M = t * group + j.
constexpr int KEY_WAVES = 4;
constexpr int KEYS_PER_KEY_ITEM = 32 * KEY_WAVES;
constexpr int ROWS_PER_ROW_TILE = 64;

// One entry of the dK/dV work list.  c < 0 marks a padding entry (the workgroup exits).
struct KeyItem {
  int32_t g;      // -1: prefix keys (seen by every row); otherwise the rollout owning the keys
  int32_t key0;   // first key of the block (prefix index, or position inside the rollout)
  int32_t c;      // kv head
  int32_t nkeys;  // keys in the block (<= KEYS_PER_KEY_ITEM)
  int32_t tile0;  // the row tiles [tile0, tile1) of the kv head this item streams (a short prefix is split over
  int32_t tile1;  //   `row_splits` items per key block to fill the chip; a rollout's own keys: see suffix_split)
  int32_t split;  // which partial-gradient slot the item writes when its pass leaves partials
  int32_t extra_tile;  // masked suffix items: one more row tile after [tile0, tile1), or -1
};

// Arguments of one attention pass (prefix or suffix).  All pointers are device pointers.
struct PassArgs {
  const void* q;        // [T, Hq, D]
  const void* k;        // prefix: [P, Hkv, D]; suffix: [T, Hkv, D]
  const void* v;
  float* o_part;        // [T, Hq, D] fp32, normalised partial output
  float* lse_part;      // [T, Hq]    fp32, natural-log LSE of the partial
  const WorkItem* items;
  const int32_t* cu;    // [G+1] packed-row offsets of the rollouts
  const void* vt;       // bf16 path: transposed-V tile images of this pass (see vt_image.hip)
  const int32_t* vt_off;  // [G+1] first tile image of each rollout (suffix pass); null for the prefix pass
  int64_t vt_tiles_per_head;  // tile images per kv head in `vt`
  int64_t num_items;
  int64_t part_rows;    // T * Hq: rows of one partial (key split s writes slot s of o_part / lse_part)
  int32_t Hq, Hkv, D, group;
  float scale;          // softmax scale
  bool causal;          // false: prefix pass (k/v indexed from 0, no mask); true: suffix pass
  // bf16 suffix pass only: finish the call in the epilogue instead of leaving a partial for the merge kernel.
  // 0: fp32 partial into o_part / lse_part; 1: no prefix, the result is final; 2: combine with the prefix
  // partial (o1, lse1).  1 and 2 write `out_final` (bf16 [T, Hq, D]) and `lse_final` ([T, Hq]).
  int32_t epilogue;
  const float* o1;
  const float* lse1;
  void* out_final;
  float* lse_final;
  // bf16 suffix pass with epilogue 1 only: sweep the prefix keys first (items carry pkeys), in the same
  // online softmax, so the call is one pass over [prefix | own keys] per block of rows.
  bool sweep_prefix;
  const void* k_pre;           // [P, Hkv, D]
  const void* vt_pre;          // prefix V tile images
  int64_t vt_pre_tiles_per_head;
  // bf16: one word per (work item, wavefront), written by the common kernel of a pass and read by its careful
  // kernel (see attn_bf16.hip); [num_items][WAVES_PER_ITEM]
  int32_t* flags;
};

struct MergeArgs {
  const float* o1;      // prefix partial (ignored when !has_prefix)
  const float* lse1;
  const float* o2;      // suffix partial
  const float* lse2;
  void* out;            // [T, Hq, D] in the plan's dtype
  float* lse;           // [T, Hq] merged
  int64_t rows;         // T * Hq
  int32_t D;
  int32_t dtype;
  bool has_prefix;
};

// Launchers; each returns a hipError_t value as int (0 = success).  `stream` is a hipStream_t.
int launch_pass_bf16(const PassArgs& a, void* stream);
int launch_pass_f32(const PassArgs& a, void* stream);
// Builds the transposed-V tile images of both passes for the bf16 path.
struct VtArgs {
  const void* v_prefix;   // [P, Hkv, D] bf16 (may be null when P == 0)
  const void* v_suffix;   // [T, Hkv, D] bf16
  void* vt_prefix;        // [Hkv][tiles_prefix][D][64] bf16 images
  void* vt_suffix;        // [Hkv][tiles_suffix][D][64] bf16 images
  const int32_t* cu;      // [G+1]
  const int32_t* vt_off;  // [G+1]
  int64_t P;
  int32_t tiles_prefix, tiles_suffix, G, Hkv, D;
  // order of the 64 keys inside a row of an image: false = as the 16 x 16 x 32 MFMAs of the forward passes deliver
  // a query's probabilities, true = as the 32 x 32 x 16 MFMAs of the backward's dQ pass deliver its dS
  bool order_32x32;
};
int launch_vt_images(const VtArgs& a, void* stream);
int launch_merge(const MergeArgs& a, void* stream);
// n-way merge of fp32 partials (see prefix_attn_merge_partials).
struct MergeNArgs {
  const float* o[PA_MAX_PARTIALS];
  const float* lse[PA_MAX_PARTIALS];
  void* out;        // [T, Hq, D] in `dtype`
  float* lse_out;   // [Hq, T] or null
  float* lse_th_out;  // [T, Hq] or null
  int64_t T;
  int32_t n, Hq, D, dtype;
};
int launch_merge_n(const MergeNArgs& a, void* stream);
int launch_lse_export(const float* lse_th, float* lse_ht, int64_t T, int32_t Hq, void* stream);
// Device address of the library's static workspace on `device` (the current device); a pa_status_t.
int static_scratch(int device, void** ptr_out);

}  // namespace pa

struct prefix_attn_plan {
  prefix_attn_desc_t desc;             // suffix_lens points into `lens`
  std::vector<int32_t> lens;           // [G]
  std::vector<int32_t> cu;             // [G+1]
  std::vector<int32_t> vt_off;         // [G+1] tile-image offsets of the rollouts (KEYS_PER_TILE keys per image)
  int64_t T = 0;
  int32_t group = 1;                   // Hq / Hkv
  int32_t num_cu = pa::NUM_CU;         // compute units the schedule is sized for
  int32_t num_xcd = pa::NUM_XCD;       // XCDs the lists are interleaved over (1: no interleaving)
  std::vector<pa::WorkItem> items[2];  // 0 = prefix pass, 1 = suffix pass
  // device-side copies (null for a host-only plan)
  int32_t* d_cu = nullptr;             // cu followed by vt_off, one allocation
  int32_t* d_vt_off = nullptr;
  int32_t tiles_prefix = 0, tiles_suffix = 0;
  int32_t key_splits = 1;              // prefix-pass items per block of rows (> 1: few rows, the prefix keys are split)
  pa::WorkItem* d_items[2] = {nullptr, nullptr};
  // backward dQ pass: the suffix list, each block of rows once per key split (split 0 also sweeps the own keys)
  std::vector<pa::WorkItem> dq_items;
  pa::WorkItem* d_dq_items = nullptr;
  // forward sweep over [prefix | own keys] (whole bf16 calls with an unsplit prefix): every block of rows once,
  // interleaved over the XCDs by kv head like the prefix pass, longest first inside a kv head
  std::vector<pa::WorkItem> sweep_items;
  pa::WorkItem* d_sweep_items = nullptr;
  // workspace layout, byte offsets
  size_t off_o1 = 0, off_o2 = 0, off_lse1 = 0, off_lse2 = 0, off_lse = 0, off_vtp = 0, off_vts = 0, off_flags = 0,
         ws_bytes = 0;
  // backward: dK/dV work lists (0 = prefix key blocks, 1 = suffix key blocks) and workspace layout
  std::vector<pa::KeyItem> key_items[2];
  pa::KeyItem* d_key_items[2] = {nullptr, nullptr};
  int64_t Mpad = 0;                    // stacked rows per kv head, rounded up to ROWS_PER_ROW_TILE
  int32_t row_splits = 1;              // items per prefix key block (> 1: fp32 partial gradients are reduced)
  // A rollout's own key block sees masked rows only near its diagonal and in the rollout's last, partly filled
  // row tile.  With suffix_split the masked kernel streams just those tiles (key_items[1]) and the mask-free
  // kernel the rest (key_items_full); both leave fp32 partials that a reduction adds.
  bool suffix_split = false;
  std::vector<pa::KeyItem> key_items_full;
  pa::KeyItem* d_key_items_full = nullptr;
  size_t boff_delta = 0, boff_lse_th = 0, boff_qs = 0, boff_dos = 0, boff_lse2s = 0, boff_deltas = 0,
         boff_toks = 0, boff_ktp = 0, boff_kts = 0, boff_part = 0, boff_dqpart = 0, bws_bytes = 0;
};
