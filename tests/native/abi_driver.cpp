// Drives the host side of the C ABI (plan building, schedule introspection, argument checks of every entry
// point) through host-only plans.  Built with -fsanitize=address,undefined against the library's host
// sources and launcher stand-ins by tests/test_host_sanitizers.py; exits non-zero on the first surprise.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <tuple>
#include <vector>

#include "prefix_attn.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "abi_driver: %s failed at line %d\n", #cond, __LINE__); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

namespace {

uint64_t rng_state = 0x9E3779B97F4A7C15ull;
uint32_t rnd(uint32_t n) {  // a small LCG: the shapes only have to vary
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33) % n;
}

prefix_attn_desc_t make_desc(int Hq, int Hkv, int D, int64_t P, const std::vector<int32_t>& lens, int dtype) {
  prefix_attn_desc_t d{};
  d.num_q_heads = Hq;
  d.num_kv_heads = Hkv;
  d.head_dim = D;
  d.prefix_len = P;
  d.num_rollouts = (int32_t)lens.size();
  d.suffix_lens = lens.data();
  d.softmax_scale = 0.125f;
  d.dtype = dtype;
  d.device = -1;
  return d;
}

void exercise(int Hq, int Hkv, int D, int64_t P, const std::vector<int32_t>& lens, int dtype) {
  prefix_attn_desc_t d = make_desc(Hq, Hkv, D, P, lens, dtype);
  prefix_attn_plan_t* plan = nullptr;
  size_t ws = 0;
  CHECK(prefix_attn_plan(&d, &plan, &ws) == PA_OK && plan);
  int64_t T = 0;
  for (int32_t s : lens) T += s;
  CHECK(prefix_attn_plan_total_tokens(plan) == T);
  int32_t rows = 0, keys = 0;
  CHECK(prefix_attn_plan_tiles(plan, &rows, &keys) == PA_OK && rows > 0 && keys > 0);
  const int group = Hq / Hkv;
  // every (rollout, block of rows, kv head) exactly once in the suffix list; the prefix ranges of a block are
  // disjoint and cover the prefix
  std::vector<int32_t> items;
  for (int pass = 0; pass < 4; ++pass) {
    const int64_t n = prefix_attn_plan_num_items(plan, pass);
    CHECK(n >= 0);
    items.assign((size_t)n * 6 + 1, -7);
    CHECK(prefix_attn_plan_items(plan, pass, items.data()) == PA_OK);
    CHECK(items[(size_t)n * 6] == -7);  // nothing written past the list
    std::map<std::tuple<int, int, int>, int64_t> covered;
    for (int64_t i = 0; i < n; ++i) {
      const int32_t* it = &items[(size_t)i * 6];
      if (it[0] < 0) continue;
      CHECK(it[0] < (int)lens.size() && it[2] >= 0 && it[2] < Hkv && it[1] % rows == 0 && it[1] < lens[it[0]] * group);
      if (pass == 0) {
        CHECK(it[4] >= 0 && it[3] > 0 && it[4] + it[3] <= P);
        covered[{it[0], it[1], it[2]}] += it[3];
      } else if (pass == 1) {
        CHECK(it[3] >= 1 && it[3] <= lens[it[0]]);
        covered[{it[0], it[1], it[2]}] += 1;
      }
    }
    int64_t blocks = 0;
    for (int32_t s : lens) blocks += ((int64_t)s * group + rows - 1) / rows;
    if (pass == 0 && P > 0) {
      CHECK((int64_t)covered.size() == blocks * Hkv);
      for (auto& kv : covered) CHECK(kv.second == P);
    }
    if (pass == 1) {
      CHECK((int64_t)covered.size() == blocks * Hkv);
      for (auto& kv : covered) CHECK(kv.second == 1);
    }
  }
  CHECK(prefix_attn_plan_num_items(plan, 4) == -1 && prefix_attn_plan_items(plan, 4, items.data()) == PA_ERR_SHAPE);
  for (int pass = 0; pass < 2; ++pass) {
    const int64_t n = prefix_attn_plan_num_key_items(plan, pass);
    CHECK(n >= 0);
    items.assign((size_t)n * 6 + 1, -7);
    CHECK(prefix_attn_plan_key_items(plan, pass, items.data()) == PA_OK && items[(size_t)n * 6] == -7);
    int64_t keys_seen = 0;
    for (int64_t i = 0; i < n; ++i) {
      const int32_t* it = &items[(size_t)i * 6];
      if (it[2] < 0) continue;
      CHECK(it[3] > 0 && it[1] >= 0);
      if (pass == 1 || it[4] == 0) keys_seen += it[3];  // a prefix block split over row ranges counts once
    }
    CHECK(keys_seen == (pass == 0 ? P : T) * Hkv);
  }
  size_t bws = 0;
  CHECK(prefix_attn_backward_workspace(plan, &bws) == PA_OK);
  // argument checks of the entry points; a host-only plan never launches
  void* p = reinterpret_cast<void*>(uintptr_t{4096});
  void* odd = reinterpret_cast<void*>(uintptr_t{4100});
  float* fp = static_cast<float*>(p);
  CHECK(prefix_attn_forward(plan, p, p, p, p, p, p, p, ws, nullptr) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_forward(plan, nullptr, p, p, p, p, p, p, ws, nullptr) == PA_ERR_NULL);
  CHECK(prefix_attn_forward(plan, odd, p, p, p, p, p, p, ws, nullptr) == PA_ERR_ALIGN);
  if (ws > 0) CHECK(prefix_attn_forward(plan, p, p, p, p, p, p, p, ws - 1, nullptr) == PA_ERR_WORKSPACE);
  CHECK(prefix_attn_forward_static(plan, p, p, p, p, p, p, nullptr, nullptr) ==
        (ws > PA_STATIC_SCRATCH_BYTES ? PA_ERR_WORKSPACE : PA_ERR_UNSUPPORTED));
  float ms[4];
  CHECK(prefix_attn_forward_timed(plan, p, p, p, p, p, p, p, ws, nullptr, nullptr) == PA_ERR_NULL);
  CHECK(prefix_attn_forward_timed(plan, p, p, p, p, p, p, p, ws, nullptr, ms) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_lse(plan, p, fp, nullptr) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_lse(plan, nullptr, fp, nullptr) == PA_ERR_NULL);
  CHECK(prefix_attn_forward_partial(plan, p, p, p, p, p, 1, fp, fp, p, ws, nullptr) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_forward_partial(plan, p, p, p, nullptr, nullptr, 0, fp, fp, p, ws, nullptr) ==
        (P > 0 ? PA_ERR_UNSUPPORTED : PA_ERR_SHAPE));
  const float* po[PA_MAX_PARTIALS + 1];
  for (auto& x : po) x = fp;
  CHECK(prefix_attn_merge_partials(plan, 0, po, po, p, nullptr, nullptr) == PA_ERR_SHAPE);
  CHECK(prefix_attn_merge_partials(plan, PA_MAX_PARTIALS + 1, po, po, p, nullptr, nullptr) == PA_ERR_SHAPE);
  CHECK(prefix_attn_merge_partials(plan, 3, po, po, p, nullptr, nullptr) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_backward(plan, p, p, p, p, p, p, p, fp, p, p, p, p, p, p, bws, nullptr) == PA_ERR_UNSUPPORTED);
  CHECK(prefix_attn_backward(plan, p, p, p, p, p, p, nullptr, fp, p, p, p, p, p, p, bws, nullptr) == PA_ERR_NULL);
  if (bws > 0)
    CHECK(prefix_attn_backward(plan, p, p, p, p, p, p, p, fp, p, p, p, p, p, p, bws - 1, nullptr) == PA_ERR_WORKSPACE);
  CHECK(prefix_attn_backward_timed(plan, p, p, p, p, p, p, p, fp, p, p, p, p, p, p, bws, nullptr, nullptr) == PA_ERR_NULL);
  prefix_attn_destroy(plan);
}

}  // namespace

int main() {
  // the benchmark configurations and the shapes the GPU tests use
  exercise(1, 1, 64, 256, {96, 96}, PA_F32);
  exercise(28, 4, 128, 4096, std::vector<int32_t>(8, 1152), PA_BF16);
  exercise(28, 4, 128, 32768, std::vector<int32_t>(8, 2304), PA_BF16);
  exercise(28, 4, 128, 230400, std::vector<int32_t>(8, 2304), PA_BF16);
  {
    std::vector<int32_t> lens;
    for (int g = 0; g < 16; ++g) lens.push_back(512 + 256 + (int32_t)rnd(3841));
    exercise(28, 4, 128, 524288, lens, PA_BF16);
  }
  exercise(28, 4, 128, 0, {32768}, PA_BF16);
  exercise(28, 4, 128, 5000, {40, 3}, PA_BF16);       // prefix key ranges
  exercise(8, 2, 64, 300, {1500, 700, 1}, PA_BF16);   // row ranges in the backward
  exercise(6, 3, 128, 300, {100, 57}, PA_BF16);       // lists not interleaved over XCDs
  exercise(3, 3, 128, 65, {1, 2, 3}, PA_F32);
  for (int i = 0; i < 200; ++i) {  // seeded random shapes
    const int Hkv = 1 + (int)rnd(4), group = 1 + (int)rnd(8), D = rnd(2) ? 64 : 128;
    const int64_t P = rnd(4) == 0 ? 0 : (int64_t)rnd(20000);
    std::vector<int32_t> lens;
    for (int g = 1 + (int)rnd(6); g > 0; --g) lens.push_back(1 + (int32_t)rnd(rnd(2) ? 40 : 3000));
    exercise(Hkv * group, Hkv, D, P, lens, rnd(4) ? PA_BF16 : PA_F32);
  }
  // descriptors that must be refused, and NULL handling
  prefix_attn_plan_t* plan = reinterpret_cast<prefix_attn_plan_t*>(uintptr_t{1});
  size_t ws = 0;
  std::vector<int32_t> lens{5, 6};
  CHECK(prefix_attn_plan(nullptr, &plan, &ws) == PA_ERR_NULL && plan == nullptr);
  auto refuse = [&](prefix_attn_desc_t d, int want) {
    prefix_attn_plan_t* q = reinterpret_cast<prefix_attn_plan_t*>(uintptr_t{1});
    CHECK(prefix_attn_plan(&d, &q, &ws) == want && q == nullptr);
  };
  prefix_attn_desc_t ok = make_desc(8, 2, 128, 100, lens, PA_BF16);
  { auto d = ok; d.num_q_heads = 7; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; d.head_dim = 96; refuse(d, PA_ERR_UNSUPPORTED); }
  { auto d = ok; d.prefix_len = -1; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; d.num_rollouts = 0; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; d.suffix_lens = nullptr; refuse(d, PA_ERR_NULL); }
  { auto d = ok; d.softmax_scale = 0.f; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; d.dtype = 9; refuse(d, PA_ERR_UNSUPPORTED); }
  { auto d = ok; d.device = -2; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; d.prefix_len = (int64_t)1 << 31; refuse(d, PA_ERR_SHAPE); }
  { auto d = ok; lens[1] = 0; refuse(d, PA_ERR_SHAPE); lens[1] = 6; }
  prefix_attn_destroy(nullptr);
  CHECK(prefix_attn_status_string(PA_ERR_ALIGN) != nullptr && prefix_attn_status_string(99) != nullptr);
  size_t lws = 0;
  CHECK(token_logprob_workspace(1000, 128, 5000, &lws) == PA_OK && lws > 0);
  CHECK(token_logprob_workspace(1000, 100, 5000, &lws) == PA_ERR_UNSUPPORTED);
  CHECK(token_logprob_workspace(1000, 128, 5000, nullptr) == PA_ERR_NULL);
  std::puts("abi_driver: ok");
  return 0;
}
