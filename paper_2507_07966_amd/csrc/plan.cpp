// Host side of the library: descriptor validation, the work lists of the two attention
// passes, workspace layout, plan lifetime and schedule introspection.
//
// Shapes follow the paper's rollout-and-prefill description (Sec. 4.2: G responses per
// question; Sec. 5.1: one cached video embedding shared by all rollouts; Sec. 5.2: prefill
// of every rollout): a shared prefix of P tokens and G ragged suffixes packed back to back.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <new>

#include "common.h"

using pa::WorkItem;

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int validate(const prefix_attn_desc_t* d) {
  if (d->num_q_heads < 1 || d->num_kv_heads < 1 || d->num_q_heads % d->num_kv_heads != 0) return PA_ERR_SHAPE;
  if (d->head_dim < 1 || d->prefix_len < 0 || d->num_rollouts < 1) return PA_ERR_SHAPE;
  if (!(d->softmax_scale > 0.0f) || !std::isfinite(d->softmax_scale)) return PA_ERR_SHAPE;
  if (d->device < -1) return PA_ERR_SHAPE;
  if (d->prefix_len > (int64_t)1 << 30) return PA_ERR_SHAPE;  // key indices are 32-bit in the kernels
  if (!d->suffix_lens) return PA_ERR_NULL;
  int64_t T = 0;
  for (int g = 0; g < d->num_rollouts; ++g) {
    if (d->suffix_lens[g] < 1) return PA_ERR_SHAPE;
    T += d->suffix_lens[g];
  }
  const int64_t group = d->num_q_heads / d->num_kv_heads;
  // stacked row indices (S_g * group) and packed rows times heads must fit 32-bit arithmetic
  for (int g = 0; g < d->num_rollouts; ++g)
    if ((int64_t)d->suffix_lens[g] * group > (int64_t)1 << 30) return PA_ERR_SHAPE;
  if (T * d->num_q_heads > (int64_t)1 << 31) return PA_ERR_SHAPE;
  if (d->dtype != PA_F32 && d->dtype != PA_BF16) return PA_ERR_UNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 128) return PA_ERR_UNSUPPORTED;
  if (d->dtype == PA_BF16) {  // the bf16 kernels address a key set (the prefix, one rollout) with 32-bit byte offsets
    const int64_t row_bytes = (int64_t)d->num_kv_heads * d->head_dim * 2, limit = (int64_t)1 << 31;
    if (d->prefix_len * row_bytes >= limit) return PA_ERR_UNSUPPORTED;
    for (int g = 0; g < d->num_rollouts; ++g)
      if (d->suffix_lens[g] * row_bytes >= limit) return PA_ERR_UNSUPPORTED;
  }
  return PA_OK;
}

// Lays per-kv-head lists out so that workgroup n (dispatched to XCD n % num_xcd) always belongs to the same
// kv head: each head owns num_xcd / Hkv XCDs, whose L2 then serves that head's tiles to all the workgroups
// walking them together.  Slots without an item hold `pad` (the workgroup exits).  When the XCD count is not
// a multiple of the head count the lists are simply concatenated.
template <class Item>
void interleave_over_xcds(const std::vector<std::vector<Item>>& per_head, int num_xcd, const Item& pad,
                          std::vector<Item>& out) {
  const int Hkv = (int)per_head.size();
  out.clear();
  if (Hkv <= num_xcd && num_xcd % Hkv == 0) {
    size_t per = 0;
    for (const auto& v : per_head) per = std::max(per, v.size());
    const int xper = num_xcd / Hkv;  // XCDs per kv head
    const size_t qlen = (per + xper - 1) / xper;
    out.assign(qlen * num_xcd, pad);
    for (int x = 0; x < num_xcd; ++x) {
      const int c = x / xper, sub = x % xper;
      for (size_t k = 0; k * xper + sub < per_head[c].size(); ++k) out[k * num_xcd + x] = per_head[c][k * xper + sub];
    }
  } else {
    for (const auto& v : per_head) out.insert(out.end(), v.begin(), v.end());
  }
}

const WorkItem PAD_ITEM{-1, 0, 0, 0, 0, 0, 0, 0};

// Prefix pass: every (kv head, rollout, block of stacked rows) sweeps all P keys.  Workgroup n
// runs on XCD n % 8 and each XCD has a private L2, so the list is interleaved such that one kv
// head's items land on a fixed subset of XCDs and walk the prefix K/V tiles together: the
// tiles are then fetched from HBM about once per XCD subset instead of once per workgroup.
//
// A call with few rows (a short prompt over a long video, say) has fewer row blocks than the
// chip has CUs.  The prefix keys are then cut into `key_splits` contiguous ranges of whole
// tiles, one item per (row block, range), each leaving its own fp32 partial; the merge combines
// them with the suffix partial.  Items of one range are adjacent so they share its tiles in L2.
void build_prefix_items(prefix_attn_plan_t& p) {
  std::vector<WorkItem>& out = p.items[0];
  out.clear();
  p.key_splits = 1;
  const int Hkv = p.desc.num_kv_heads;
  const int P = (int)p.desc.prefix_len;
  if (P == 0) return;
  int64_t blocks = 0;
  for (int g = 0; g < p.desc.num_rollouts; ++g)
    blocks += ((int64_t)p.lens[g] * p.group + pa::ROWS_PER_ITEM - 1) / pa::ROWS_PER_ITEM;
  blocks *= Hkv;
  if (p.desc.dtype == PA_BF16) {  // one round of workgroups, at least 8 tiles per range
    const int64_t fit = p.num_cu / blocks, by_len = p.tiles_prefix / 8;
    p.key_splits = (int32_t)std::max<int64_t>(1, std::min<int64_t>({fit, by_len, PA_MAX_PARTIALS - 1}));
  }
  const int tiles_per_split = (p.tiles_prefix + p.key_splits - 1) / p.key_splits;
  p.key_splits = (p.tiles_prefix + tiles_per_split - 1) / tiles_per_split;  // no empty range
  const int KS = p.key_splits;
  std::vector<std::vector<WorkItem>> per_head(Hkv);
  for (int c = 0; c < Hkv; ++c)
    for (int s = 0; s < KS; ++s) {
      const int key0 = std::min(s * tiles_per_split * pa::KEYS_PER_TILE, P);
      const int key1 = std::min((s + 1) * tiles_per_split * pa::KEYS_PER_TILE, P);
      for (int g = 0; g < p.desc.num_rollouts; ++g) {
        const int nrows = p.lens[g] * p.group;
        for (int row0 = 0; row0 < nrows; row0 += pa::ROWS_PER_ITEM)
          per_head[c].push_back({g, row0, c, key1 - key0, key0, s, 0, 0});
      }
    }
  interleave_over_xcds(per_head, p.num_xcd, PAD_ITEM, out);
}

// Suffix pass: a block of stacked rows needs the rollout's keys 0..(position of its last row).
// Items are issued longest first so the ragged, triangular work packs well.
void build_suffix_items(prefix_attn_plan_t& p) {
  std::vector<WorkItem>& out = p.items[1];
  out.clear();
  for (int c = 0; c < p.desc.num_kv_heads; ++c)
    for (int g = 0; g < p.desc.num_rollouts; ++g) {
      const int nrows = p.lens[g] * p.group;
      for (int row0 = 0; row0 < nrows; row0 += pa::ROWS_PER_ITEM) {
        const int last_row = std::min(row0 + pa::ROWS_PER_ITEM, nrows) - 1;
        out.push_back({g, row0, c, last_row / p.group + 1, 0, 0, 0, 0});
      }
    }
  std::stable_sort(out.begin(), out.end(), [](const WorkItem& a, const WorkItem& b) { return a.nkeys > b.nkeys; });
}

// Backward, dQ pass: the suffix pass's blocks of rows (longest first); each sweeps the prefix and
// then its own keys.  With key splits (few rows, see build_prefix_items) a block appears once per
// prefix key range; split 0 also sweeps the own keys, and the fp32 partial dQ are added afterwards.
void build_dq_items(prefix_attn_plan_t& p) {
  p.dq_items.clear();
  const int P = (int)p.desc.prefix_len;
  const int KS = p.key_splits;
  const int tiles_per_split = (p.tiles_prefix + KS - 1) / KS;  // the ranges of build_prefix_items
  for (int s = 0; s < KS; ++s) {
    const int key0 = std::min(s * tiles_per_split * pa::KEYS_PER_TILE, P);
    const int key1 = std::min((s + 1) * tiles_per_split * pa::KEYS_PER_TILE, P);
    for (const WorkItem& it : p.items[1])
      p.dq_items.push_back({it.g, it.row0, it.c, s == 0 ? it.nkeys : 0, key0, s, key1 - key0, 0});
  }
  // An unsplit prefix: lay the blocks out over the XCDs by kv head like the prefix pass, so that the
  // workgroups of an XCD walk the same K, V and K^T tiles together (-0.4 % at a 32K prefix, -1.5 % at 230K).
  const int Hkv = p.desc.num_kv_heads;
  if (KS == 1 && P > 0 && Hkv <= p.num_xcd && p.num_xcd % Hkv == 0) {
    std::vector<std::vector<WorkItem>> per_head(Hkv);
    for (const WorkItem& it : p.dq_items) per_head[it.c].push_back(it);  // longest first inside a kv head
    interleave_over_xcds(per_head, p.num_xcd, PAD_ITEM, p.dq_items);
  }
}

// Forward sweep (one pass over [prefix | own keys] per block of rows): the prefix dominates, so the blocks are
// laid out like the prefix pass's (one kv head per subset of XCDs, sharing its K/V tiles in that L2), and
// inside a kv head longest first.
void build_sweep_items(prefix_attn_plan_t& p) {
  p.sweep_items.clear();
  const int Hkv = p.desc.num_kv_heads;
  const int P = (int)p.desc.prefix_len;
  if (P == 0 || p.key_splits != 1 || p.desc.dtype != PA_BF16 || p.tiles_prefix > pa::SWEEP_MAX_PREFIX_TILES) return;
  std::vector<std::vector<WorkItem>> per_head(Hkv);
  for (const WorkItem& it : p.items[1]) per_head[it.c].push_back({it.g, it.row0, it.c, it.nkeys, 0, 0, P, 0});  // sorted already
  interleave_over_xcds(per_head, p.num_xcd, PAD_ITEM, p.sweep_items);
}

// Backward, dK/dV pass: one item per block of KEYS_PER_KEY_ITEM keys of a kv head.  A prefix
// block streams the stacked rows of every rollout, all blocks of a kv head in the same order,
// so (as in the prefix pass) one kv head's blocks are kept on a fixed subset of XCDs and share
// the streamed Q/dO tiles through that subset's L2.  A suffix block streams the rollout's rows
// from its first key on; longest first.
void build_key_items(prefix_attn_plan_t& p) {
  const int Hkv = p.desc.num_kv_heads;
  const int P = (int)p.desc.prefix_len;
  const int KB = pa::KEYS_PER_KEY_ITEM;
  std::vector<pa::KeyItem>& pre = p.key_items[0];
  pre.clear();
  p.row_splits = 1;
  if (P > 0) {
    // One workgroup per CU runs at a time and all items of a launch take equally long, so the launch
    // takes ceil(items / CUs) rounds.  Few key blocks (a short prefix) leave CUs idle, and a count
    // just above a multiple of the CU count pays a whole round for its tail.  Splitting the streamed
    // rows over R items per key block shortens the rounds; it costs a prologue/epilogue per item
    // (about 3 tile steps) and, for R > 1, writing and re-reading fp32 partials (about 0.03 tile
    // steps per item).  Take the R that minimises this estimate; keep R = 1 unless it gains 2 %.
    const int64_t row_tiles = p.Mpad / pa::ROWS_PER_ROW_TILE;
    const int64_t blocks = (int64_t)Hkv * ((P + KB - 1) / KB);
    auto cost = [&](int64_t r) {
      const int64_t rounds = (blocks * r + p.num_cu - 1) / p.num_cu;
      return (double)rounds * ((double)((row_tiles + r - 1) / r) + 3.0) + (r > 1 ? 0.03 * (double)(blocks * r) : 0.0);
    };
    int64_t R = 1;
    double best = 0.98 * cost(1);
    for (int64_t r = 2; r <= 16 && row_tiles / r >= 64; ++r)
      if (cost(r) < best) {
        best = cost(r);
        R = r;
      }
    p.row_splits = (int32_t)R;
    const int64_t per_split = (row_tiles + R - 1) / R;
    std::vector<std::vector<pa::KeyItem>> per_head(Hkv);
    for (int c = 0; c < Hkv; ++c)
      for (int key0 = 0; key0 < P; key0 += KB)
        for (int r = 0; r < (int)R; ++r) {
          const int32_t t0 = (int32_t)std::min<int64_t>(r * per_split, row_tiles);
          const int32_t t1 = (int32_t)std::min<int64_t>((r + 1) * per_split, row_tiles);
          per_head[c].push_back({-1, key0, c, std::min(KB, P - key0), t0, t1, r, 0});
        }
    interleave_over_xcds(per_head, p.num_xcd, pa::KeyItem{-1, 0, -1, 0, 0, 0, 0, 0}, pre);
  }
  // A rollout's own key blocks.  Row r (position i) sees key j of its rollout iff i >= j, so a block of keys
  // [key0, key0 + n) needs the mask only on the rows at positions key0 .. key0 + n - 2 (the diagonal) and in
  // the rollout's last row tile when that tile also holds rows of the next rollout; every tile between is
  // fully visible.  Long rollouts (bf16) therefore run as two items per block: the masked kernel on the
  // diagonal tiles plus that last tile, the mask-free kernel on the tiles between, each leaving fp32 partial
  // gradients that a reduction adds.  The mask-free items walk their tiles from the rollout's end backwards:
  // all blocks of a rollout share that end, so the blocks running at the same time stream the same Q/dO tiles
  // and share them in L2, where the masked kernel, which starts every block at its own diagonal, fetched
  // 40 GB per launch for a 32,768-token sequence.  Short rollouts keep one masked item per block.
  std::vector<pa::KeyItem>& suf = p.key_items[1];
  std::vector<pa::KeyItem>& full = p.key_items_full;
  suf.clear();
  full.clear();
  const int RT = pa::ROWS_PER_ROW_TILE;
  struct Ranges { int32_t tile_b, tile_full, tile_e_full, tile_e; };
  auto ranges = [&](int g, int key0, int n) {
    const int64_t m_begin = (int64_t)(p.cu[g] + key0) * p.group;
    const int64_t m_full = (int64_t)(p.cu[g] + key0 + n - 1) * p.group;  // first row that sees the whole block
    const int64_t m_end = (int64_t)p.cu[g + 1] * p.group;
    return Ranges{(int32_t)(m_begin / RT), (int32_t)((m_full + RT - 1) / RT), (int32_t)(m_end / RT),
                  (int32_t)((m_end + RT - 1) / RT)};
  };
  // Worth it for long rollouts only (measured: a 32,768-token sequence -4 ... -9 % on the pass depending on the
  // box, a 230,400-token one -6.7 %, 2,304-token rollouts +8 %: two launches, partials and a reduction for little
  // mask-free work).
  constexpr int SPLIT_MIN_TILES = 512;
  p.suffix_split = false;
  if (p.desc.dtype == PA_BF16)
    for (int g = 0; g < p.desc.num_rollouts && !p.suffix_split; ++g) {
      const Ranges r = ranges(g, 0, std::min(KB, p.lens[g]));
      p.suffix_split = r.tile_e_full - r.tile_full >= SPLIT_MIN_TILES;  // a rollout's first block has the longest mask-free range
    }
  for (int c = 0; c < Hkv; ++c)
    for (int g = 0; g < p.desc.num_rollouts; ++g)
      for (int key0 = 0; key0 < p.lens[g]; key0 += KB) {
        const int n = std::min(KB, p.lens[g] - key0);
        const Ranges r = ranges(g, key0, n);
        if (p.suffix_split && r.tile_e_full > r.tile_full) {
          suf.push_back({g, key0, c, n, r.tile_b, r.tile_full, 0, r.tile_e_full < r.tile_e ? r.tile_e_full : -1});
          // the mask-free kernel indexes keys over all packed tokens: key0 is the packed token index here
          full.push_back({-2, p.cu[g] + key0, c, n, r.tile_full, r.tile_e_full, 1, -1});
        } else {
          suf.push_back({g, key0, c, n, r.tile_b, r.tile_e, 0, -1});
          if (p.suffix_split) full.push_back({-1, p.cu[g] + key0, c, n, 0, 0, 1, -1});  // no tiles: writes zeros
        }
      }
  auto tiles_of = [](const pa::KeyItem& a) { return a.tile1 - a.tile0 + (a.extra_tile >= 0 ? 1 : 0); };
  std::stable_sort(suf.begin(), suf.end(), [&](const pa::KeyItem& a, const pa::KeyItem& b) { return tiles_of(a) > tiles_of(b); });
  std::stable_sort(full.begin(), full.end(), [&](const pa::KeyItem& a, const pa::KeyItem& b) { return tiles_of(a) > tiles_of(b); });
  if (!full.empty()) {  // one kv head per subset of XCDs, longest first inside a head (-1.3 % on the pass)
    std::vector<std::vector<pa::KeyItem>> per_head(Hkv);
    for (const pa::KeyItem& it : full) per_head[it.c].push_back(it);
    interleave_over_xcds(per_head, p.num_xcd, pa::KeyItem{-1, 0, -1, 0, 0, 0, 0, -1}, full);
  }
}

// Backward workspace: delta and the re-ordered LSE (used by the fp32 path); for bf16 also the stacked Q/dO copies, the
// per-row statistics and the transposed K images.
void layout_backward_workspace(prefix_attn_plan_t& p) {
  const prefix_attn_desc_t& d = p.desc;
  const size_t rows = (size_t)p.T * d.num_q_heads;
  p.Mpad = ((int64_t)p.T * p.group + pa::ROWS_PER_ROW_TILE - 1) / pa::ROWS_PER_ROW_TILE * pa::ROWS_PER_ROW_TILE;
  p.boff_delta = 0;
  p.boff_lse_th = align_up(rows * sizeof(float), 256);
  size_t end = 2 * p.boff_lse_th;
  if (d.dtype == PA_BF16) {
    const size_t stacked = align_up((size_t)d.num_kv_heads * p.Mpad * d.head_dim * 2, 256);
    const size_t stats = align_up((size_t)d.num_kv_heads * p.Mpad * 4, 256);
    const size_t image = (size_t)d.head_dim * pa::KEYS_PER_TILE * 2;
    p.boff_qs = end;
    p.boff_dos = p.boff_qs + stacked;
    p.boff_lse2s = p.boff_dos + stacked;
    p.boff_deltas = p.boff_lse2s + stats;
    p.boff_toks = p.boff_deltas + stats;
    p.boff_ktp = p.boff_toks + stats;
    p.boff_kts = p.boff_ktp + align_up((size_t)d.num_kv_heads * p.tiles_prefix * image, 256);
    end = p.boff_kts + align_up((size_t)d.num_kv_heads * p.tiles_suffix * image, 256);
    // fp32 partial dK, dV: of the prefix per row split [2][row_splits][P][Hkv][D]; of the rollouts' own keys, when
    // their pass is split into a masked and a mask-free item per block, [2][2][T][Hkv][D].  The two stages run
    // one after the other and share the region.
    p.boff_part = end;
    size_t part = 0;
    if (p.row_splits > 1) part = (size_t)2 * p.row_splits * d.prefix_len * d.num_kv_heads * d.head_dim * sizeof(float);
    if (p.suffix_split) part = std::max(part, (size_t)2 * 2 * p.T * d.num_kv_heads * d.head_dim * sizeof(float));
    end += align_up(part, 256);
    p.boff_dqpart = end;  // fp32 partial dQ per key split: [key_splits][T][Hq][D]
    if (p.key_splits > 1) end += align_up((size_t)p.key_splits * rows * d.head_dim * sizeof(float), 256);
  }
  p.bws_bytes = end;
}

}  // namespace

extern "C" {

int prefix_attn_plan(const prefix_attn_desc_t* desc, prefix_attn_plan_t** plan_out, size_t* workspace_bytes_out) {
  if (plan_out) *plan_out = nullptr;
  if (!desc || !plan_out || !workspace_bytes_out) return PA_ERR_NULL;
  const int st = validate(desc);
  if (st != PA_OK) return st;
  prefix_attn_plan_t* p = new (std::nothrow) prefix_attn_plan_t();
  if (!p) return PA_ERR_ALLOC;
  if (desc->device >= 0) {  // size the schedule for the device it will run on
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, desc->device) != hipSuccess || cus < 1) {
      (void)hipGetLastError();
      delete p;
      return PA_ERR_HIP;
    }
    if (cus != pa::NUM_CU) {  // not the layout the XCD interleaving is built for
      p->num_cu = cus;
      p->num_xcd = 1;
    }
  }
  try {
    p->desc = *desc;
    p->lens.assign(desc->suffix_lens, desc->suffix_lens + desc->num_rollouts);
    p->desc.suffix_lens = p->lens.data();
    p->cu.assign(desc->num_rollouts + 1, 0);
    for (int g = 0; g < desc->num_rollouts; ++g) p->cu[g + 1] = p->cu[g] + p->lens[g];
    p->T = p->cu.back();
    p->vt_off.assign(desc->num_rollouts + 1, 0);
    for (int g = 0; g < desc->num_rollouts; ++g)
      p->vt_off[g + 1] = p->vt_off[g] + (p->lens[g] + pa::KEYS_PER_TILE - 1) / pa::KEYS_PER_TILE;
    p->tiles_suffix = p->vt_off.back();
    p->tiles_prefix = (int32_t)((desc->prefix_len + pa::KEYS_PER_TILE - 1) / pa::KEYS_PER_TILE);
    p->group = desc->num_q_heads / desc->num_kv_heads;
    build_prefix_items(*p);
    build_suffix_items(*p);
    build_dq_items(*p);
    build_sweep_items(*p);
    p->Mpad = ((int64_t)p->T * p->group + pa::ROWS_PER_ROW_TILE - 1) / pa::ROWS_PER_ROW_TILE * pa::ROWS_PER_ROW_TILE;
    build_key_items(*p);
  } catch (const std::bad_alloc&) {
    delete p;
    return PA_ERR_ALLOC;
  }
  const size_t rows = (size_t)p->T * desc->num_q_heads;
  const size_t o_bytes = align_up(rows * desc->head_dim * sizeof(float), 256);
  const size_t l_bytes = align_up(rows * sizeof(float), 256);
  const size_t ks = (size_t)p->key_splits;  // the prefix pass leaves one partial per key split
  p->off_o1 = 0;
  p->off_o2 = ks * o_bytes;
  p->off_lse1 = (ks + 1) * o_bytes;
  p->off_lse2 = p->off_lse1 + ks * l_bytes;
  p->off_lse = p->off_lse2 + l_bytes;
  p->off_vtp = p->off_lse + l_bytes;
  size_t end = p->off_vtp;
  if (desc->dtype == PA_BF16) {  // transposed-V tile images, bf16 path only
    const size_t image = (size_t)desc->head_dim * pa::KEYS_PER_TILE * 2;
    p->off_vts = p->off_vtp + align_up((size_t)desc->num_kv_heads * p->tiles_prefix * image, 256);
    end = p->off_vts + align_up((size_t)desc->num_kv_heads * p->tiles_suffix * image, 256);
    // one word per (work item, wavefront) of the longest work list: a pass's common kernel tells its careful
    // kernel which items to redo; the passes run one after the other and share the region
    const size_t items = std::max({p->items[0].size(), p->items[1].size(), p->sweep_items.size()});
    p->off_flags = end;
    end += align_up(items * pa::WAVES_PER_ITEM * sizeof(int32_t), 256);
  }
  p->ws_bytes = end;
  layout_backward_workspace(*p);

  if (desc->device >= 0) {
    int prev = 0;
    bool ok = hipGetDevice(&prev) == hipSuccess && hipSetDevice(desc->device) == hipSuccess;
    if (ok) {
      const size_t n = p->cu.size();
      ok = hipMalloc((void**)&p->d_cu, 2 * n * sizeof(int32_t)) == hipSuccess &&
           hipMemcpy(p->d_cu, p->cu.data(), n * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
           hipMemcpy(p->d_cu + n, p->vt_off.data(), n * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
      p->d_vt_off = p->d_cu + n;
      for (int s = 0; ok && s < 2; ++s) {
        if (p->items[s].empty()) continue;
        const size_t bytes = p->items[s].size() * sizeof(WorkItem);
        ok = hipMalloc((void**)&p->d_items[s], bytes) == hipSuccess &&
             hipMemcpy(p->d_items[s], p->items[s].data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
      }
      if (ok && !p->sweep_items.empty()) {
        const size_t bytes = p->sweep_items.size() * sizeof(WorkItem);
        ok = hipMalloc((void**)&p->d_sweep_items, bytes) == hipSuccess &&
             hipMemcpy(p->d_sweep_items, p->sweep_items.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
      }
      if (ok && !p->dq_items.empty()) {
        const size_t bytes = p->dq_items.size() * sizeof(WorkItem);
        ok = hipMalloc((void**)&p->d_dq_items, bytes) == hipSuccess &&
             hipMemcpy(p->d_dq_items, p->dq_items.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
      }
      for (int s = 0; ok && s < 2; ++s) {
        if (p->key_items[s].empty()) continue;
        const size_t bytes = p->key_items[s].size() * sizeof(pa::KeyItem);
        ok = hipMalloc((void**)&p->d_key_items[s], bytes) == hipSuccess &&
             hipMemcpy(p->d_key_items[s], p->key_items[s].data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
      }
      // set-up for prefix_attn_forward_static: look its workspace up now, with the plan's device current,
      // so that the call itself only reads a table
      void* unused = nullptr;
      ok = ok && pa::static_scratch(desc->device, &unused) == PA_OK;
      if (ok && !p->key_items_full.empty()) {
        const size_t bytes = p->key_items_full.size() * sizeof(pa::KeyItem);
        ok = hipMalloc((void**)&p->d_key_items_full, bytes) == hipSuccess &&
             hipMemcpy(p->d_key_items_full, p->key_items_full.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
      }
      (void)hipSetDevice(prev);
    }
    if (!ok) {
      (void)hipGetLastError();
      prefix_attn_destroy(p);
      return PA_ERR_ALLOC;
    }
  }
  *plan_out = p;
  *workspace_bytes_out = p->ws_bytes;
  return PA_OK;
}

void prefix_attn_destroy(prefix_attn_plan_t* plan) {
  if (!plan) return;
  if (plan->d_cu) (void)hipFree(plan->d_cu);
  for (int s = 0; s < 2; ++s)
    if (plan->d_items[s]) (void)hipFree(plan->d_items[s]);
  for (int s = 0; s < 2; ++s)
    if (plan->d_key_items[s]) (void)hipFree(plan->d_key_items[s]);
  if (plan->d_key_items_full) (void)hipFree(plan->d_key_items_full);
  if (plan->d_dq_items) (void)hipFree(plan->d_dq_items);
  if (plan->d_sweep_items) (void)hipFree(plan->d_sweep_items);
  delete plan;
}

const char* prefix_attn_status_string(int status) {
  switch (status) {
    case PA_OK: return "ok";
    case PA_ERR_NULL: return "a required pointer is NULL";
    case PA_ERR_SHAPE: return "a size is out of range or inconsistent";
    case PA_ERR_UNSUPPORTED: return "valid but unsupported configuration";
    case PA_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case PA_ERR_WORKSPACE: return "workspace too small";
    case PA_ERR_ALLOC: return "allocation failed";
    case PA_ERR_HIP: return "HIP runtime call or kernel launch failed";
    default: return "unknown status";
  }
}

int prefix_attn_plan_tiles(const prefix_attn_plan_t* plan, int32_t* rows_per_item, int32_t* keys_per_tile) {
  if (!plan || !rows_per_item || !keys_per_tile) return PA_ERR_NULL;
  *rows_per_item = pa::ROWS_PER_ITEM;
  *keys_per_tile = pa::KEYS_PER_TILE;
  return PA_OK;
}

int64_t prefix_attn_plan_num_items(const prefix_attn_plan_t* plan, int32_t pass) {
  if (!plan || pass < 0 || pass > 3) return -1;
  return (int64_t)(pass == 3 ? plan->sweep_items : pass == 2 ? plan->dq_items : plan->items[pass]).size();
}

int prefix_attn_plan_items(const prefix_attn_plan_t* plan, int32_t pass, int32_t* items_out) {
  if (!plan || !items_out) return PA_ERR_NULL;
  if (pass < 0 || pass > 3) return PA_ERR_SHAPE;
  const std::vector<WorkItem>& v = pass == 3 ? plan->sweep_items : pass == 2 ? plan->dq_items : plan->items[pass];
  for (size_t n = 0; n < v.size(); ++n) {
    items_out[6 * n + 0] = v[n].g;
    items_out[6 * n + 1] = v[n].row0;
    items_out[6 * n + 2] = v[n].c;
    items_out[6 * n + 3] = v[n].nkeys;
    items_out[6 * n + 4] = v[n].key0;
    items_out[6 * n + 5] = v[n].pkeys;
  }
  return PA_OK;
}

int64_t prefix_attn_plan_total_tokens(const prefix_attn_plan_t* plan) { return plan ? plan->T : -1; }

int prefix_attn_backward_workspace(const prefix_attn_plan_t* plan, size_t* workspace_bytes_out) {
  if (!plan || !workspace_bytes_out) return PA_ERR_NULL;
  *workspace_bytes_out = plan->bws_bytes;
  return PA_OK;
}

int64_t prefix_attn_plan_num_key_items(const prefix_attn_plan_t* plan, int32_t pass) {
  if (!plan || pass < 0 || pass > 2) return -1;
  return (int64_t)(pass == 2 ? plan->key_items_full : plan->key_items[pass]).size();
}

int prefix_attn_plan_key_items(const prefix_attn_plan_t* plan, int32_t pass, int32_t* items_out) {
  if (!plan || !items_out) return PA_ERR_NULL;
  if (pass < 0 || pass > 2) return PA_ERR_SHAPE;
  const std::vector<pa::KeyItem>& v = pass == 2 ? plan->key_items_full : plan->key_items[pass];
  for (size_t n = 0; n < v.size(); ++n) {
    items_out[6 * n + 0] = v[n].g;
    items_out[6 * n + 1] = v[n].key0;
    items_out[6 * n + 2] = v[n].c;
    items_out[6 * n + 3] = v[n].nkeys;
    items_out[6 * n + 4] = v[n].tile0;
    items_out[6 * n + 5] = v[n].tile1;
  }
  return PA_OK;
}

int prefix_attn_plan_key_item_extra_tiles(const prefix_attn_plan_t* plan, int32_t pass, int32_t* tiles_out) {
  if (!plan || !tiles_out) return PA_ERR_NULL;
  if (pass < 0 || pass > 2) return PA_ERR_SHAPE;
  const std::vector<pa::KeyItem>& v = pass == 2 ? plan->key_items_full : plan->key_items[pass];
  for (size_t n = 0; n < v.size(); ++n) tiles_out[n] = pass == 1 ? v[n].extra_tile : -1;
  return PA_OK;
}

}  // extern "C"
