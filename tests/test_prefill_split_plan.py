"""How prompt chunks are cut into workgroups (host logic, no GPU): fsf_plan_prefill_groups."""
import numpy as np
import pytest

from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl


def plan(seqs, H=40, cus=256, window=0):
    cfg = fsf.make_cfg(H, H, 128, 64, "bf16", 1 << 20, window=window)
    return fsf.plan_prefill_groups(cfg, wl.make_descs(seqs), cus)


def tiles_of(seqs):
    """(sequence, first row, one past last row) of every 256-row tile, in tile order.  Chunks of at
    most two slices of 16 rows (one query head per KV head here) run on the streaming kernel."""
    out = []
    for s, (n, c) in enumerate(seqs):
        if n > 32:
            out += [(s, i0, min(i0 + 256, n)) for i0 in range(0, n, 256)]
    return out


def check_partition(groups, n_tiles):
    """every tile once if unsplit, else each of its parts exactly once; slabs dense and unique"""
    seen = {}
    slabs = []
    for tile, part, n_parts, slab in groups.tolist():
        assert 0 <= tile < n_tiles and 0 <= part < n_parts
        seen.setdefault(tile, []).append((part, n_parts))
        if n_parts == 1:
            assert slab == -1
        else:
            slabs.append(slab)
    assert sorted(seen) == list(range(n_tiles))
    for tile, parts in seen.items():
        n = parts[0][1]
        assert sorted(p for p, _ in parts) == list(range(n)) and all(q == n for _, q in parts)
    assert sorted(slabs) == list(range(len(slabs)))
    return {t: p[0][1] for t, p in seen.items()}


def test_one_long_chunk_whole_rounds_are_left_alone():
    """4096 rows x 32 heads = 512 workgroups = two full rounds of 256 units: nothing to split"""
    g = plan([(4096, 8192)], H=32)
    assert g.shape[0] == 16 and np.all(g[:, 2] == 1)
    assert g[:, 0].tolist() == list(range(15, -1, -1))      # most keys first


def test_partial_last_round_is_filled():
    """4096 rows x 40 heads = 640 workgroups = 2.5 rounds: the 128 of the last round (4 tiles, rounded
    up to whole tiles) are cut in two; they are the lightest tiles and start last"""
    g = plan([(4096, 8192)], H=40)
    parts = check_partition(g, 16)
    assert [parts[t] for t in range(16)] == [2] * 4 + [1] * 12
    assert g[:12, 0].tolist() == list(range(15, 3, -1))
    assert g[12:, 0].tolist() == [3, 3, 2, 2, 1, 1, 0, 0]


def test_remainder_of_a_prompt_over_its_long_prefix_is_cut_and_starts_first():
    """what a SplitFuse pass looks like when a prompt ends: its last 64 rows (20000 tokens cached,
    314 steps) next to the first 3900 rows of the next prompt (at most 61 steps per tile); spread
    evenly a unit would work 131 steps, so the remainder is cut into 3 parts"""
    seqs = [(64, 20000), (3900, 0)]
    g = plan(seqs, H=40)
    parts = check_partition(g, 17)
    assert parts[0] == 3 and g[:3, 0].tolist() == [0, 0, 0] and g[:3, 3].tolist() == [0, 1, 2]
    assert g[3, 0] == 16                                     # then the next prompt's tiles, most keys first


def test_less_than_one_round_every_tile_that_outlasts_the_even_share_is_cut():
    """one 64-row chunk at 3000 cached tokens, 64 heads: 64 workgroups of 48 steps on 256 units;
    the even share is 12 steps, so the tile is cut into 4"""
    g = plan([(64, 3000)], H=64)
    assert g.tolist() == [[0, 0, 4, 0], [0, 1, 4, 1], [0, 2, 4, 2], [0, 3, 4, 3]]


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_partition(seed):
    rng = np.random.default_rng(900 + seed)
    seqs = []
    for _ in range(int(rng.integers(1, 7))):
        seqs.append((int(rng.integers(2, 3000)), int(rng.choice([0, 0, 100, 5000, 30000]))))
    seqs += [(1, int(rng.integers(0, 4000))) for _ in range(int(rng.integers(0, 5)))]
    rng.shuffle(seqs)
    seqs = [tuple(int(x) for x in s) for s in seqs]
    H = int(rng.choice([1, 8, 32, 40, 64]))
    cus = int(rng.choice([16, 64, 256, 304]))
    window = int(rng.choice([0, 0, 700, 4096]))
    g = plan(seqs, H=H, cus=cus, window=window)
    n_tiles = len(tiles_of(seqs))
    parts = check_partition(g, n_tiles)
    assert sum(n for n in parts.values() if n > 1) * H <= 512          # the partial-result buffer's bound
    # no part shorter than 8 steps
    cfgw = window
    for t, (s, i0, i1) in enumerate(tiles_of(seqs)):
        c = seqs[s][1]
        lo = max(0, c + i0 - cfgw + 1) if cfgw else 0
        steps = (c + i1 - 1 - (lo & ~63)) // 64 + 1
        assert steps // parts[t] >= 8 or parts[t] == 1


def test_short_chunks_are_not_tiled():
    """chunks that fit two streaming slices (32 rows at one query head per KV head, 8 rows at four)
    leave the tiled kernel; the limit is a tuning field"""
    seqs = [(32, 5000), (33, 5000), (2, 0), (1, 9)]
    assert sorted(set(plan(seqs, H=8)[:, 0].tolist())) == [0]            # only the 33-row chunk
    def plan_with(hq, hkv, tuning=None):
        cfg = fsf.make_cfg(hq, hkv, 128, 64, "bf16", 1 << 20, tuning=tuning)
        return len(set(fsf.plan_prefill_groups(cfg, wl.make_descs([(8, 100), (9, 100), (40, 0)]), 256)[:, 0].tolist()))
    assert plan_with(8, 2) == 2                                           # 4 rows per slice: 9 and 40 rows are tiled
    assert plan_with(8, 2, fsf.Tuning(stream_chunk_slices=-1)) == 3
    assert plan_with(8, 2, fsf.Tuning(stream_chunk_slices=3)) == 1
    assert plan_with(8, 2, fsf.Tuning(stream_chunk_slices=16)) == 0


def test_a_lone_remainder_fills_one_round_and_no_more():
    """64 rows over 20000 cached tokens, 40 heads: 40 workgroups; 6 parts make 240, a 7th would
    start a second round"""
    g = plan([(64, 20000)], H=40)
    assert g[:, 2].tolist() == [6] * 6
