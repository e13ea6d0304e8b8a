"""Pins of the oracle's queue schedule: what the paper states about the FIFO block queue."""
import os

import pytest

from oracle.schedule import blockwise_schedule, bubble_ratio_reverse, bubble_ratio_sequential

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def by_step(sched):
    out = {}
    for e in sched:
        out.setdefault(e["step"], []).append(e)
    return out


def test_bubble_worked_example():
    for N, T, B, pct in rows("bubble_ratio.txt"):
        r = bubble_ratio_reverse(int(N), int(T), int(B))
        assert r == pytest.approx(11 / 211)
        assert round(100 * r, 1) == float(pct)
    # reverse order beats sequential order (appendix); ratio vanishes as the video grows
    assert bubble_ratio_reverse(4, 50, 4) < bubble_ratio_sequential(4, 50, 4) == pytest.approx(15 / 215)
    assert bubble_ratio_reverse(4, 50, 1000) < 1e-3
    # N > Block_num form, as printed: N=4, T=50, Block_num=3 -> (3*(4-50)+4*48+1) = 55
    assert bubble_ratio_reverse(4, 50, 3) == pytest.approx(55 / (55 + 150))


def test_queue_worked_example():
    for N, T, B, first_full, last_full, first_pop, total in rows("queue_example.txt"):
        N, T, B = int(N), int(T), int(B)
        s = blockwise_schedule(T, B, num_b=8, num_c=8)
        assert len(s) == int(total) == B * T
        steps = by_step(s)
        assert sorted(steps) == list(range(1, T + B))
        full = [st for st, es in steps.items() if len(es) >= N]
        assert min(full) == int(first_full) and max(full) == int(last_full)
        # block 1 is processed for the last time (level 1) at step T: it pops after step T
        last_of_b1 = max(e["step"] for e in s if e["block"] == 1)
        assert last_of_b1 == int(first_pop)
        assert [e for e in s if e["block"] == 1 and e["step"] == last_of_b1][0]["level"] == 1


@pytest.mark.parametrize("T,B", [(8, 8), (50, 4), (5, 12), (3, 1)])
def test_queue_invariants(T, B):
    s = blockwise_schedule(T, B, num_b=4, num_c=4, t_max=1000.0)
    assert len(s) == T * B
    for st, es in by_step(s).items():
        blocks = [e["block"] for e in es]
        levels = [e["level"] for e in es]
        assert blocks == sorted(blocks, reverse=True)                 # tail (latest block) first
        assert levels == sorted(levels, reverse=True)                 # noisiest first ...
        assert all(a - b == 1 for a, b in zip(levels, levels[1:]))    # ... one level apart, strictly decreasing
        assert all(b2 == b1 - 1 for b1, b2 in zip(blocks, blocks[1:]))
        assert es[0]["cache_block"] == 0                               # the tail block has no cache source
        for prev, e in zip(es, es[1:]):
            assert e["cache_block"] == prev["block"] == e["block"] + 1
            assert (e["cache_first"], e["cache_frames"]) == (0, 2)
    for b in range(1, B + 1):
        mine = [e for e in s if e["block"] == b]
        assert [e["level"] for e in mine] == list(range(T, 0, -1))     # every level exactly once, in order
        assert mine[0]["step"] == b                                    # enters at step b at the top level
        assert all(e["timestep"] == 1000.0 * e["level"] / T for e in mine)
        assert all(e["frame0"] == 4 * (b - 1) and e["n_frames"] == 4 for e in mine)


def test_single_block_is_plain_loop():
    s = blockwise_schedule(5, 1, num_b=4, num_c=4)
    assert [(e["step"], e["level"], e["cache_block"]) for e in s] == [(i + 1, 5 - i, 0) for i in range(5)]


def test_linear_timesteps_of_queue_config():
    s = blockwise_schedule(8, 8, num_b=4, num_c=4, t_max=1000.0)
    assert sorted({e["timestep"] for e in s}, reverse=True) == [1000.0, 875.0, 750.0, 625.0, 500.0, 375.0, 250.0, 125.0]
    full = [e for e in s if e["step"] == 8]
    assert [e["timestep"] for e in full] == [1000.0, 875.0, 750.0, 625.0, 500.0, 375.0, 250.0, 125.0]


def test_longer_first_block_and_sequential_order():
    s = blockwise_schedule(4, 3, num_b=4, num_c=2, first_block_frames=5)
    f = {e["block"]: (e["frame0"], e["n_frames"]) for e in s}
    assert f == {1: (0, 5), 2: (5, 4), 3: (9, 4)}
    q = blockwise_schedule(4, 3, num_b=4, num_c=2, first_block_frames=5, order="sequential")
    assert len(q) == 12
    for st, es in by_step(q).items():
        assert [e["block"] for e in es] == sorted(e["block"] for e in es)      # head first
        assert es[0]["cache_block"] == 0
        for prev, e in zip(es, es[1:]):
            assert e["cache_block"] == prev["block"] == e["block"] - 1
            assert e["cache_first"] == prev["n_frames"] - 1 and e["cache_frames"] == 1
    # 257 latent frames in 4-frame blocks with a 5-frame first block -> 64 blocks
    long = blockwise_schedule(2, 64, num_b=4, num_c=4, first_block_frames=5)
    last = max(long, key=lambda e: e["frame0"])
    assert last["frame0"] + last["n_frames"] == 257


def _abs_frames(first, n):
    return set(range(first, first + n))


@pytest.mark.parametrize("order", ["reverse", "sequential"])
@pytest.mark.parametrize("T,block_num,num_b,num_c,first", [(4, 5, 4, 4, 6), (3, 4, 8, 8, None), (6, 3, 2, 4, 4), (2, 6, 3, 2, None)])
def test_extended_block_and_feature_cache(T, block_num, num_b, num_c, first, order):
    """Sec. 3.2: with the feature cache the input shrinks from [B_{i-1}, B_i, B_{i+1}] to [B_{i-1}, B_i] and the
    cached K/V are exactly the frames that were dropped."""
    blk = blockwise_schedule(T, block_num, num_b, num_c, first, order=order)
    ext = blockwise_schedule(T, block_num, num_b, num_c, first, order=order, variant="extended")
    noc = blockwise_schedule(T, block_num, num_b, num_c, first, order=order, variant="nocache")
    assert len(blk) == len(ext) == len(noc) == T * block_num
    half = num_c // 2
    total = (first or num_b) + (block_num - 1) * num_b
    by_key = {(e["step"], e["block"]): e for e in ext}
    for b0, e, n in zip(blk, ext, noc):
        for k in ("step", "block", "level", "timestep", "frame0", "n_frames"):
            assert b0[k] == e[k] == n[k]
        assert (b0["in_frame0"], b0["in_frames"], b0["keep_first"]) == (b0["frame0"], b0["n_frames"], 0)
        for x in (e, n):
            own = _abs_frames(x["in_frame0"] + x["keep_first"], x["n_frames"])
            assert own == _abs_frames(x["frame0"], x["n_frames"])              # the block sits at keep_first
            assert 0 <= x["in_frame0"] and x["in_frame0"] + x["in_frames"] <= total
        assert n["cache_block"] == 0 and n["in_frames"] <= n["n_frames"] + num_c
        assert e["in_frames"] <= e["n_frames"] + half                          # the reduced input of Sec. 3.2
        cached = set()
        if e["cache_block"]:
            src = by_key[(e["step"], e["cache_block"])]
            assert src["block"] == e["block"] + (1 if order == "reverse" else -1)
            assert 0 <= e["cache_first"] and e["cache_first"] + e["cache_frames"] <= src["in_frames"]
            cached = _abs_frames(src["in_frame0"] + e["cache_first"], e["cache_frames"])
            assert cached <= _abs_frames(src["frame0"], src["n_frames"])      # the neighbour's own frames
            assert b0["cache_frames"] == e["cache_frames"]
        # fed frames + cached frames = what is fed without the cache
        assert _abs_frames(e["in_frame0"], e["in_frames"]) | cached == _abs_frames(n["in_frame0"], n["in_frames"])
        assert not _abs_frames(e["in_frame0"], e["in_frames"]) & cached


def test_extended_block_example_by_hand():
    # T = 2, 3 blocks of 4 frames, Num_C = 4, tail to head.  Step 2 holds blocks 2 and 1 (block 3 is not there
    # yet): block 2 is fed [frames 2,3 of block 1 ; block 2] = frames 2..7, no cache; block 1 is fed alone
    # (it has no earlier neighbour) and reads the K/V of block 2's first two frames, which sit at offset 2 of
    # that pass's input.  Without the cache block 1 is fed frames 0..5.
    ext = [e for e in blockwise_schedule(2, 3, 4, 4, variant="extended") if e["step"] == 2]
    assert [(e["block"], e["in_frame0"], e["in_frames"], e["keep_first"], e["cache_block"], e["cache_first"], e["cache_frames"])
            for e in ext] == [(2, 2, 6, 2, 0, 0, 0), (1, 0, 4, 0, 2, 2, 2)]
    noc = [e for e in blockwise_schedule(2, 3, 4, 4, variant="nocache") if e["step"] == 2]
    assert [(e["block"], e["in_frame0"], e["in_frames"], e["keep_first"]) for e in noc] == [(2, 2, 6, 2), (1, 0, 6, 0)]
    # step 3: blocks 3 and 2 (block 1 has left the queue and no longer counts as a neighbour); block 3 is fed
    # [frames 6,7 ; block 3], block 2 is fed alone and reads block 3's first two frames at offset 2
    ext3 = [e for e in blockwise_schedule(2, 3, 4, 4, variant="extended") if e["step"] == 3]
    assert [(e["block"], e["in_frame0"], e["in_frames"], e["keep_first"], e["cache_block"], e["cache_first"], e["cache_frames"])
            for e in ext3] == [(3, 6, 6, 2, 0, 0, 0), (2, 4, 4, 0, 3, 2, 2)]
