"""CPU-only tests of the C-ABI library: it loads, exports what the header declares,
rejects bad arguments before any launch, and its schedule covers every visible
(query row, key) pair exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_07966_amd as pa
from tests.random_shapes import random_shapes
from paper_2507_07966_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "prefix_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:prefix_attn|token_logprob|grpo)_\w+)\s*\(", header))
    assert {"prefix_attn_plan", "prefix_attn_forward", "prefix_attn_lse", "prefix_attn_destroy"} <= declared
    lib = ctypes.CDLL(binding.library_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTED_SYMBOLS) | set(binding.EXPORTED_SYMBOLS_OTHER)


def host_plan(**kw):
    args = dict(num_q_heads=28, num_kv_heads=4, head_dim=128, prefix_len=4096, suffix_lens=[1152] * 8,
                softmax_scale=128 ** -0.5, dtype="bf16", device=-1)
    args.update(kw)
    return pa.prefix_attn_plan(**args)


@pytest.mark.parametrize("kw,status", [
    (dict(num_q_heads=0), 2), (dict(num_kv_heads=3), 2), (dict(prefix_len=-1), 2), (dict(suffix_lens=[]), 2),
    (dict(suffix_lens=[5, 0, 3]), 2), (dict(softmax_scale=0.0), 2), (dict(softmax_scale=float("nan")), 2),
    (dict(softmax_scale=float("inf")), 2), (dict(head_dim=96), 3), (dict(dtype=7), 3), (dict(device=-2), 2),
    (dict(prefix_len=(1 << 30) + 1), 2),
])
def test_plan_rejects_bad_descriptors(kw, status):
    with pytest.raises(pa.PrefixAttnError) as e:
        host_plan(**kw)
    assert e.value.status == status


def test_null_arguments_and_status_strings():
    lib = binding.load_library()
    assert lib.prefix_attn_plan(None, None, None) == 1
    assert lib.prefix_attn_forward(None, None, None, None, None, None, None, None, 0, None) == 1
    assert lib.prefix_attn_lse(None, None, None, None) == 1
    lib.prefix_attn_destroy(None)
    assert lib.prefix_attn_plan_num_items(None, 0) == -1
    for s in range(8):
        assert pa.prefix_attn_status_string(s) not in ("", "unknown status")
    assert pa.prefix_attn_status_string(99) == "unknown status"


def test_forward_checks_arguments_before_launch():
    """With a host-only plan nothing can be launched; the checks must fire in order without touching memory."""
    plan = host_plan()
    lib = binding.load_library()
    a = 0x10000  # fake, 16-byte aligned "device" addresses: never dereferenced by the checks
    f = lambda *p: lib.prefix_attn_forward(plan.handle, *p)
    big = plan.workspace_bytes
    assert f(None, a, a, a, a, a, a, big, None) == 1
    assert f(a, None, a, a, a, a, a, big, None) == 1          # prefix needed when P > 0
    assert f(a, a, a, a, a, a, None, big, None) == 1
    assert f(a + 8, a, a, a, a, a, a, big, None) == 4
    assert f(a, a, a, a, a + 2, a, a, big, None) == 4
    assert f(a, a, a, a, a, a, a, big - 1, None) == 5
    assert f(a, a, a, a, a, a, a, big, None) == 3             # host-only plan cannot launch
    assert lib.prefix_attn_lse(plan.handle, a, a + 4, None) == 4
    assert lib.prefix_attn_lse(plan.handle, a, a, None) == 3
    noprefix = host_plan(prefix_len=0)
    assert lib.prefix_attn_forward(noprefix.handle, a, None, None, a, a, a, a, noprefix.workspace_bytes, None) == 3


def test_workspace_size_matches_layout():
    plan = host_plan()
    T, Hq, D = 1152 * 8, 28, 128
    assert plan.total_tokens == T
    need = 2 * T * Hq * D * 4 + 3 * T * Hq * 4
    images = 4 * (4096 // 64 + 8 * (1152 // 64)) * D * 64 * 2     # bf16: transposed-V tile images
    flags = max(len(plan.items(w)) for w in (0, 1, 3)) * 8 * 4      # bf16: one word per (work item, wavefront)
    assert need + images + flags <= plan.workspace_bytes <= need + images + flags + 8 * 256
    f32 = host_plan(dtype="f32")
    assert need <= f32.workspace_bytes <= need + 5 * 256


def coverage(plan, Hq, Hkv, P, lens):
    """Count how often each (kv head, rollout, stacked row) is covered by each pass and check key extents."""
    r = Hq // Hkv
    bm, bn = plan.tiles()
    assert bm > 0 and bn > 0
    for which in (0, 1):
        items = plan.items(which)
        seen = [[np.zeros(S * r, dtype=np.int64) for S in lens] for _ in range(Hkv)]
        ranges = {}
        for g, row0, c, nkeys, key0, pkeys in items:
            assert pkeys == 0
            if g < 0:
                continue
            assert 0 <= g < len(lens) and 0 <= c < Hkv and row0 % bm == 0
            n = lens[g] * r
            assert row0 < n
            hi = min(row0 + bm, n)
            if which == 0:                               # the prefix rectangle, no mask; possibly in key ranges
                assert key0 % bn == 0 and nkeys > 0
                ranges.setdefault((c, g, row0), []).append((key0, key0 + nkeys))
            else:
                seen[c][g][row0:hi] += 1
                assert key0 == 0
                last_pos = (hi - 1) // r
                assert nkeys == last_pos + 1             # keys 0..position of the item's last row
                assert nkeys <= lens[g]
        if which == 0 and P == 0:
            assert len(items) == 0
            continue
        if which == 0:                                   # the key ranges of a block of rows tile [0, P)
            for (c, g, row0), rs in ranges.items():
                rs.sort()
                assert rs[0][0] == 0 and rs[-1][1] == P and all(a[1] == b[0] for a, b in zip(rs, rs[1:]))
                seen[c][g][row0:min(row0 + bm, lens[g] * r)] += 1
        for c in range(Hkv):
            for g in range(len(lens)):
                assert (seen[c][g] == 1).all(), (which, c, g)
    # the backward's dQ list: every block of rows of the suffix list, its prefix key ranges tiling [0, P) and
    # its own keys swept by exactly one of its items
    blocks = {}
    for g, row0, c, nkeys, key0, pkeys in plan.items(2):
        if g < 0:
            continue
        assert key0 % bn == 0
        blocks.setdefault((g, row0, c), []).append((key0, key0 + pkeys, nkeys))
    suffix = {(g, row0, c): nk for g, row0, c, nk, _, _ in plan.items(1) if g >= 0}
    assert set(blocks) == set(suffix)
    for key, rs in blocks.items():
        rs.sort()
        assert rs[0][0] == 0 and rs[-1][1] == P and all(a[1] == b[0] for a, b in zip(rs, rs[1:]))
        assert all(b > a for a, b, _ in rs) or P == 0
        assert sorted(nk for _, _, nk in rs) == [0] * (len(rs) - 1) + [suffix[key]]


@pytest.mark.parametrize("Hq,Hkv,P,lens", [
    (28, 4, 4096, [1152] * 8), (28, 4, 100, [1, 37, 300, 5]), (4, 4, 0, [70, 3]), (8, 1, 64, [64]),
    (6, 3, 1000, [257, 256, 255]), (16, 16, 130, [33] * 5),
    (28, 4, 32768, [256]), (28, 4, 1000, [5, 3]), (8, 2, 70000, [40, 1, 17]),      # few rows: prefix keys are split
])
def test_schedule_covers_every_pair_exactly_once(Hq, Hkv, P, lens):
    plan = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, prefix_len=P, suffix_lens=lens)
    coverage(plan, Hq, Hkv, P, lens)


@pytest.mark.parametrize("Hq,Hkv,D,P,lens", random_shapes())
def test_schedule_covers_random_shapes(Hq, Hkv, D, P, lens):
    plan = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, prefix_len=P, suffix_lens=list(lens))
    coverage(plan, Hq, Hkv, P, list(lens))
    key_coverage(plan, Hq, Hkv, P, list(lens))


def test_single_sweep_list_only_for_short_unsplit_prefixes():
    """Whole bf16 calls with a prefix of at most 1,024 tiles run one sweep per block of rows: the list holds every
    block of the suffix list once, with the whole prefix, one kv head per XCD subset."""
    plan = host_plan()                                                                  # P = 4,096: 64 tiles
    sweep, suffix = plan.items(3), plan.items(1)
    real = sweep[sweep[:, 0] >= 0]
    assert sorted(map(tuple, real[:, :4].tolist())) == sorted(map(tuple, suffix[:, :4].tolist()))
    assert (real[:, 4] == 0).all() and (real[:, 5] == 4096).all()
    for x in range(8):
        assert len({int(it[2]) for it in sweep[x::8] if it[0] >= 0}) == 1
    assert len(host_plan(prefix_len=32768, suffix_lens=[2304] * 8).items(3)) == 2016    # 512 tiles: still one sweep
    assert len(host_plan(prefix_len=230400, suffix_lens=[2304] * 8).items(3)) == 0      # 3,600 tiles: separate passes
    assert len(host_plan(prefix_len=4096, suffix_lens=[256]).items(3)) == 0             # few rows: key ranges instead
    assert len(host_plan(dtype="f32").items(3)) == 0
    assert len(host_plan(prefix_len=0).items(3)) == 0


def test_few_rows_split_the_prefix_keys_and_size_the_workspace():
    """28 blocks of rows for 256 CUs: 9 key ranges per block (one round of workgroups), one fp32 partial each."""
    Hq, Hkv, D, P, S = 28, 4, 128, 32768, 256
    plan = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, prefix_len=P, suffix_lens=[S])
    items = plan.items(0)
    real = items[items[:, 0] >= 0]
    assert len(real) == 28 * 9
    assert sorted(set(real[:, 4].tolist())) == [i * 57 * 64 for i in range(9)]      # 512 tiles in ranges of 57
    rows = S * Hq
    partials = (9 + 1) * rows * D * 4 + (9 + 2) * rows * 4
    images = Hkv * (P // 64 + S // 64) * D * 64 * 2
    flags = max(len(plan.items(w)) for w in (0, 1, 3)) * 8 * 4      # one word per (work item, wavefront)
    assert partials + images + flags <= plan.workspace_bytes <= partials + images + flags + 25 * 256
    # the backward keeps one fp32 partial dQ per key range on top of its unsplit layout
    one = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, prefix_len=7 * 64, suffix_lens=[S])   # 7 tiles: no split
    extra_tiles = Hkv * (P // 64 - 7) * D * 64 * 2
    grown = plan.backward_workspace_bytes - one.backward_workspace_bytes - extra_tiles
    assert 9 * rows * D * 4 <= grown <= 9 * rows * D * 4 + 512
    f32 = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, prefix_len=P, suffix_lens=[S], dtype="f32")
    assert len(f32.items(0)) == 28 + 4                                              # fp32 path: no key splits (32 = 8 XCD queues x 4)


def test_prefix_items_are_grouped_by_kv_head_per_xcd():
    """Workgroup n runs on XCD n % 8: with 4 kv heads each XCD must only ever see one kv head."""
    plan = host_plan()
    items = plan.items(0)
    for x in range(8):
        heads = {int(it[2]) for it in items[x::8] if it[0] >= 0}
        assert len(heads) == 1
    # suffix pass is issued longest first
    nk = plan.items(1)[:, 3]
    assert (np.diff(nk) <= 0).all()


def test_c5_ragged_plan_builds_fast():
    rng = np.random.default_rng(0)
    lens = (512 + rng.integers(256, 4097, size=16)).tolist()
    plan = host_plan(prefix_len=8192 * 64, suffix_lens=lens)
    coverage(plan, 28, 4, 8192 * 64, lens)


# ---------------------------------------------------------------- backward: schedule and argument checks

def key_coverage(plan, Hq, Hkv, P, lens):
    """Every (prefix key, row tile) pair and every suffix key of every kv head lies in exactly one dK/dV work item."""
    row_tiles = -(-sum(lens) * (Hq // Hkv) // 64)
    pre = [np.zeros((P, row_tiles), dtype=np.int32) for _ in range(Hkv)]
    for g, key0, c, n, t0, t1 in plan.key_items(0):
        if c < 0:
            continue
        assert g == -1 and 0 < n <= 128 and key0 % 128 == 0 and key0 + n <= P and 0 <= t0 <= t1 <= row_tiles
        pre[c][key0:key0 + n, t0:t1] += 1
    suf = [[np.zeros(S, dtype=np.int32) for S in lens] for _ in range(Hkv)]
    for g, key0, c, n, _, _ in plan.key_items(1):
        assert 0 <= g < len(lens) and 0 <= c < Hkv and 0 < n <= 128 and key0 % 128 == 0 and key0 + n <= lens[g]
        suf[c][g][key0:key0 + n] += 1
    for c in range(Hkv):
        assert (pre[c] == 1).all()
        for g in range(len(lens)):
            assert (suf[c][g] == 1).all()
    suffix_tile_coverage(plan, Hq // Hkv, Hkv, lens)


def suffix_tile_coverage(plan, group, Hkv, lens):
    """The rollouts' own key blocks: the tiles of the masked item (its range and its extra tile) and of the
    mask-free item (when the plan splits the pass) together are exactly the row tiles from the block's first key
    to the rollout's end, each once; every row of a mask-free tile lies in the block's rollout and sees all of
    the block's keys."""
    off = np.concatenate([[0], np.cumsum(lens)])
    masked, extra, free = plan.key_items(1), plan.key_item_extra_tiles(1), plan.key_items(2)
    split = len(free) > 0
    assert not split or (free[:, 2] >= 0).sum() == len(masked)
    seen = {}
    for (g, key0, c, n, t0, t1), x in zip(masked.tolist(), extra.tolist()):
        tiles = list(range(t0, t1)) + ([x] if x >= 0 else [])
        assert len(set(tiles)) == len(tiles)
        seen[(c, int(off[g]) + key0)] = tiles
    for g_, pkey0, c, n, t0, t1 in free.tolist():
        if c < 0:
            continue
        assert g_ in (-1, -2)
        g = int(np.searchsorted(off, pkey0, side="right") - 1)
        key0 = pkey0 - int(off[g])
        for t in range(t0, t1):
            rows = np.arange(64 * t, 64 * t + 64)                       # stacked rows M = token * group + head
            tok = rows // group
            assert (tok >= off[g] + key0 + n - 1).all() and (tok < off[g + 1]).all()
        assert not set(range(t0, t1)) & set(seen[(c, pkey0)])
        seen[(c, pkey0)] += list(range(t0, t1))
    for (g, key0, c, n, _, _) in masked.tolist():
        first = (int(off[g]) + key0) * group // 64
        last = -(-int(off[g + 1]) * group // 64)
        assert sorted(seen[(c, int(off[g]) + key0)]) == list(range(first, last)), (g, key0, c)


@pytest.mark.parametrize("Hq,Hkv,P,lens", [
    (28, 4, 4096, [1152] * 8), (28, 4, 100, [1, 37, 300, 5]), (4, 4, 0, [70, 3]), (6, 3, 1000, [257, 256, 255]),
    (2, 2, 129, [513]), (8, 2, 300, [1500, 700, 1]), (28, 4, 0, [4700, 33]), (7, 1, 64, [130, 127, 5000, 129]),
    (4, 1, 7, [9000, 8300, 1]),
])
def test_backward_schedule_covers_every_key_once(Hq, Hkv, P, lens):
    plan = host_plan(num_q_heads=Hq, num_kv_heads=Hkv, prefix_len=P, suffix_lens=lens)
    key_coverage(plan, Hq, Hkv, P, lens)


def test_long_rollouts_split_their_own_key_blocks_into_masked_and_mask_free_items():
    plan = host_plan(prefix_len=0, suffix_lens=[8192, 100])        # 896 row tiles in the long sequence: split
    masked, free = plan.key_items(1), plan.key_items(2)
    real = free[free[:, 2] >= 0]
    assert len(real) == len(masked) == 4 * (64 + 1)
    assert (masked[:, 5] - masked[:, 4]).max() <= 16               # 127 positions x 7 heads = 14 tiles of diagonal (+ edges)
    assert (real[:, 5] - real[:, 4]).max() == 896 - 14             # the first block of the sequence: all tiles after its diagonal
    assert (real[:, 0] == -2).sum() == 4 * 63                      # these walk backwards; the rest stream no tile
    assert len(host_plan().key_items(2)) == 0                      # rollouts of 1,152 tokens keep one masked item per block
    f32 = host_plan(prefix_len=0, suffix_lens=[8192], dtype="f32")
    assert len(f32.key_items(2)) == 0
    assert plan.backward_workspace_bytes >= 2 * 2 * 8292 * 4 * 128 * 4      # holds the two partial-gradient slots [2][2][T][Hkv][D]


def test_backward_items_are_grouped_by_kv_head_per_xcd():
    plan = host_plan()
    items = plan.key_items(0)
    for x in range(8):
        heads = {int(it[2]) for it in items[x::8] if it[2] >= 0}
        assert len(heads) == 1
    k1 = plan.key_items(1)
    work = k1[:, 5] - k1[:, 4] + (plan.key_item_extra_tiles(1) >= 0)
    assert (np.diff(work) <= 0).all()          # suffix key blocks: most row tiles first


def test_backward_workspace_and_argument_checks():
    plan = host_plan()
    lib = binding.load_library()
    T, Hq, Hkv, D, P = 1152 * 8, 28, 4, 128, 4096
    mpad = -(-T * (Hq // Hkv) // 64) * 64
    stacked = 2 * Hkv * mpad * D * 2                       # Q and dO gathered into stacked-row order
    images = Hkv * (P // 64 + 8 * (1152 // 64)) * D * 64 * 2
    splits = len([1 for it in plan.key_items(0) if it[2] == 0 and it[1] == 0])     # items of one key block
    assert splits == 2                                                              # 128 key blocks -> 256 items, one round
    partials = 2 * splits * P * Hkv * D * 4            # (rollouts this short keep one masked item per own key block)
    need = 2 * T * Hq * 4 + stacked + 3 * Hkv * mpad * 4 + images + partials
    assert need <= plan.backward_workspace_bytes <= need + 12 * 256
    c3 = host_plan(prefix_len=32768, suffix_lens=[2304] * 8)
    assert len(c3.key_items(0)) == 1024                                             # 4 full rounds of 256: no split
    tail = host_plan(prefix_len=32768 + 256, suffix_lens=[2048] * 8)               # 1032 blocks: 8 would pay a fifth round
    assert len(tail.key_items(0)) == 1032 * 7
    assert host_plan(dtype="f32").backward_workspace_bytes <= 2 * T * Hq * 4 + 2 * 256
    a = 0x10000
    big = plan.backward_workspace_bytes

    def call(**kw):
        args = dict(q=a, kp=a, vp=a, ks=a, vs=a, out=a, do=a, lse=a, dq=a, dkp=a, dvp=a, dks=a, dvs=a, ws=a, n=big)
        args.update(kw)
        return lib.prefix_attn_backward(plan.handle, *[args[k] for k in
                                        ("q", "kp", "vp", "ks", "vs", "out", "do", "lse", "dq", "dkp", "dvp", "dks", "dvs", "ws", "n")], None)

    assert lib.prefix_attn_backward(None, *([a] * 14), big, None) == 1
    for name in ("q", "ks", "vs", "out", "do", "lse", "dq", "dks", "dvs", "ws", "kp", "dvp"):
        assert call(**{name: None}) == 1, name
    assert call(do=a + 8) == 4 and call(dkp=a + 4) == 4
    assert call(n=big - 1) == 5
    assert call() == 3                                      # host-only plan cannot launch
    noprefix = host_plan(prefix_len=0)
    st = lib.prefix_attn_backward(noprefix.handle, a, None, None, a, a, a, a, a, a, None, None, a, a, a,
                                  noprefix.backward_workspace_bytes, None)
    assert st == 3
    n = ctypes.c_size_t()
    assert lib.prefix_attn_backward_workspace(None, ctypes.byref(n)) == 1
    assert lib.prefix_attn_plan_num_key_items(None, 0) == -1


def test_sharded_calls_check_arguments():
    plan = host_plan()
    lib = binding.load_library()
    a = 0x10000
    big = plan.workspace_bytes
    fp = lambda *p: lib.prefix_attn_forward_partial(plan.handle, *p)
    assert fp(a, a, a, a, a, 1, a, None, a, big, None) == 1          # the partial's LSE is required
    assert fp(a, a, a, None, a, 1, a, a, a, big, None) == 1          # suffix keys needed when included
    assert fp(a, a, a, None, None, 0, a, a, a, big, None) == 3       # prefix-only: suffix may be NULL; host-only plan
    assert fp(a, a, a, a, a, 1, a, a + 4, a, big, None) == 4
    noprefix = host_plan(prefix_len=0)
    assert lib.prefix_attn_forward_partial(noprefix.handle, a, None, None, None, None, 0, a, a, a,
                                           noprefix.workspace_bytes, None) == 2   # a partial over no keys
    ptrs = (ctypes.c_void_p * 17)(*([a] * 17))
    mp = lambda n, o=ptrs, l=ptrs, out=a, lse=a: lib.prefix_attn_merge_partials(plan.handle, n, o, l, out, lse, None)
    assert mp(0) == 2 and mp(17) == 2
    assert mp(2, None) == 1 and mp(2, out=None) == 1
    holes = (ctypes.c_void_p * 2)(a, None)
    assert mp(2, holes) == 1
    odd = (ctypes.c_void_p * 2)(a, a + 8)
    assert mp(2, ptrs, odd) == 4
    assert mp(3) == 3 and mp(3, lse=None) == 3                        # host-only plan cannot launch


def test_logprob_calls_check_arguments():
    lib = binding.load_library()
    a = 0x10000
    assert pa.token_logprob_workspace(1000, 3584, 152064) >= 594 * 1000 * 8 + 1000 * 4
    n = ctypes.c_size_t()
    assert lib.token_logprob_workspace(0, 64, 10, ctypes.byref(n)) == 2
    assert lib.token_logprob_workspace(5, 100, 10, ctypes.byref(n)) == 3          # hidden_dim not a multiple of 64
    assert lib.token_logprob_workspace(5, 64, 10, None) == 1
    big = pa.token_logprob_workspace(5, 64, 10)
    f = lambda *p: lib.token_logprob_forward(*p)
    assert f(None, a, a, 5, 64, 10, 1.0, a, None, a, big, None) == 1
    assert f(a, a, a, 5, 64, 10, 0.0, a, None, a, big, None) == 2
    assert f(a, a, a, 5, 64, 10, float("nan"), a, None, a, big, None) == 2
    assert f(a, a + 2, a, 5, 64, 10, 1.0, a, None, a, big, None) == 4
    assert f(a, a, a, 5, 64, 10, 1.0, a, None, a, big - 1, None) == 5
    assert lib.grpo_group_advantages(None, 8, 1, a, None) == 1
    assert lib.grpo_group_advantages(a, 0, 1, a, None) == 2


def test_loading_the_library_first_does_not_bring_in_a_second_hip_runtime():
    """In a fresh process, load the library before anything imports torch: exactly one copy of the HIP
    runtime may be mapped afterwards (torch carries its own; a second one cannot allocate on the device)."""
    import subprocess
    import sys
    code = ("import paper_2507_07966_amd as pa; pa.load_library(); import torch; "
            "m = open('/proc/self/maps').read(); "
            "print(len({l.split()[-1] for l in m.splitlines() if 'libamdhip64' in l}))")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip() == "1"


def test_bf16_key_sets_of_2_gib_are_unsupported():
    """The bf16 kernels address the prefix (and each rollout) with 32-bit byte offsets: 2 GiB of K rows is refused
    at plan time, just below passes; fp32 plans have no such limit."""
    rows = (1 << 31) // (4 * 128 * 2)                       # 2,097,152 tokens at Hkv = 4, D = 128
    with pytest.raises(pa.PrefixAttnError) as e:
        host_plan(prefix_len=rows, suffix_lens=[8])
    assert e.value.status == 3
    with pytest.raises(pa.PrefixAttnError) as e:
        host_plan(prefix_len=64, suffix_lens=[rows])
    assert e.value.status == 3
    host_plan(prefix_len=rows - 1, suffix_lens=[8])
