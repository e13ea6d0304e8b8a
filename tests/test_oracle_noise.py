"""Pins of the oracle's coordinated noise initialisation: the properties Sec. 3.3 states, a hand-worked
example, and brute force over every word sequence of a tiny case."""
import itertools
import os

import numpy as np
import pytest

from oracle.noise import gather_frames, noise_assignment

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_examples():
    with open(os.path.join(GOLD, "noise_example.txt")) as f:
        lines = [ln for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(lines) == 2
    for ln in lines:
        head, words, blocks = [p.strip() for p in ln.split("|")]
        num_b, num_c, n = map(int, head.split())
        want = [[int(v) for v in b.split()] for b in blocks.split("/")]
        assert noise_assignment(n, num_b, num_c, [int(w) for w in words.split()]) == want


@pytest.mark.parametrize("num_b,num_c,block_num", [(4, 4, 8), (4, 2, 5), (8, 8, 6), (3, 6, 7), (5, 0, 4), (1, 2, 4)])
@pytest.mark.parametrize("seed", [0, 1])
def test_properties_the_section_states(num_b, num_c, block_num, seed):
    rng = np.random.default_rng(seed)
    words = rng.integers(0, 2**32, size=block_num * max(num_b, 1), dtype=np.uint64)
    blocks = noise_assignment(block_num, num_b, num_c, words)
    half, pool = num_c // 2, num_b + num_c // 2
    assert [len(b) for b in blocks] == [pool] + [num_b] * (block_num - 1)      # the first block is longer
    assert blocks[0] == list(range(pool))                                     # ... and is the whole pool
    for b, blk in enumerate(blocks):
        assert len(set(blk)) == len(blk) and all(0 <= p < pool for p in blk)    # no noise twice inside a block
        if b:
            tail = blocks[b - 1][len(blocks[b - 1]) - half:] if half else []
            assert not set(tail) & set(blk)             # nor together with the frames it is concatenated with
            assert set(tail) | set(blk) == set(range(pool))                   # the rest of the pool, all of it
    assert set().union(*blocks) == set(range(pool))                           # the complete pool stays in use


def test_brute_force_every_word_sequence():
    # Num_B = 3, Num_C = 2, 3 blocks: 2 words per later block, each word only matters mod 3 / mod 2
    seen = set()
    for w in itertools.product(range(3), range(2), range(3), range(2)):
        blocks = noise_assignment(3, 3, 2, list(w))
        assert blocks[0] == [0, 1, 2, 3]
        assert sorted(blocks[1]) == [0, 1, 2]                     # pool minus the first block's last frame
        assert sorted(blocks[2]) == sorted(set(range(4)) - {blocks[1][-1]})
        seen.add((tuple(blocks[1]), tuple(blocks[2])))
    # every one of the 3! orders of block 2 occurs, each with 3! orders of block 3
    assert len({s[0] for s in seen}) == 6 and len(seen) == 36


def test_shuffle_is_not_degenerate():
    rng = np.random.default_rng(7)
    counts = {}
    for _ in range(6000):
        blk = noise_assignment(2, 3, 2, rng.integers(0, 2**32, size=2, dtype=np.uint64))[1]
        counts[tuple(blk)] = counts.get(tuple(blk), 0) + 1
    assert len(counts) == 6 and min(counts.values()) > 800         # 1000 expected per order


def test_gather_is_a_frame_copy():
    pool = np.arange(5 * 6, dtype=np.float64).reshape(5, 2, 3)
    out = gather_frames(pool, [4, 0, 4])
    assert out.shape == (3, 2, 3)
    assert (out[0] == pool[4]).all() and (out[1] == pool[0]).all() and (out[2] == pool[4]).all()
