"""Oracle of the coordinated noise initialisation (TEST INFRASTRUCTURE).

Paper Sec. 3.3 and the overview figure's caption: all blocks draw their initial noise from one shared
pool of frame noises.  The first block uses the whole pool and is Num_C/2 frames longer than the others,
so the pool holds Num_B + Num_C/2 frame noises.  Every later block is initialised from the pool frames
that were NOT used by the last Num_C/2 frames of the block initialised before it (the queue's tail);
those candidates are shuffled and become the new block's frames.  Consequences the paper states: no
noise is repeated inside a block together with the neighbouring frames it is concatenated with, and the
whole pool stays in use throughout.

Readings where the paper is silent: the first block takes the pool in its stored order; candidates are
listed in ascending pool index before the shuffle; the shuffle is the Fisher-Yates walk from the last
position down, position i exchanging with position (word mod (i + 1)), one 32-bit random word per
exchange, words consumed in order (Num_B - 1 words per later block).  The random words are an input.
"""
import numpy as np


def noise_assignment(block_num, num_b, num_c, words):
    """Pool-frame index of every frame of every block.

    Returns a list of block_num lists: block 1 has num_b + num_c // 2 entries, the others num_b.
    `words` is a sequence of at least (block_num - 1) * (num_b - 1) unsigned 32-bit integers."""
    half = num_c // 2
    assert half <= num_b, "the excluded noises are those of a block's last Num_C/2 frames (Sec. 3.3); it has Num_B"
    pool = num_b + half
    blocks = [list(range(pool))]
    pos = 0
    for _ in range(1, block_num):
        prev = blocks[-1]
        excluded = set(prev[len(prev) - half:]) if half else set()
        cand = [p for p in range(pool) if p not in excluded]
        assert len(cand) == num_b
        for i in range(num_b - 1, 0, -1):
            j = int(words[pos]) % (i + 1)
            pos += 1
            cand[i], cand[j] = cand[j], cand[i]
        blocks.append(cand)
    return blocks


def gather_frames(pool, index):
    """Initial noise of one block: pool is [pool_frames, ...], index the block's pool-frame indices."""
    return np.stack([pool[i] for i in index], axis=0)
