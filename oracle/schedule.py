"""Oracle of the block-wise denoising queue and the bubble-ratio closed forms (TEST INFRASTRUCTURE).

Queue (paper Sec. 3.1): the video is cut into Block_num temporal blocks; one new
block enters the FIFO queue's tail at the highest noise level at each diffusion
step, every block in the queue is processed once per step from tail (noisiest)
to head (cleanest), every processed block drops one noise level, and the head
leaves the queue once it is clean.  Feature cache (Sec. 3.2): a block reuses the
self-attention K/V of the block processed immediately before it in the same
step; the paper's extended block additionally feeds the Num_C/2 touching frames
of the other neighbour along with the block, and without the cache both
neighbours' frames are fed.  First block is longer by Num_C/2 frames (Sec. 3.3).
"""


def blockwise_schedule(T, block_num, num_b, num_c, first_block_frames=None, t_max=1000.0, order="reverse",
                       variant="block"):
    """List of block passes in execution order.  Each pass is a dict:
    step (1-based diffusion step), block (1-based, video order), level (T..1), timestep,
    frame0, n_frames (the block itself), in_frame0, in_frames (the frames fed to the model), keep_first
    (offset of the block's own frames inside the input), cache_block (0 = none), cache_first, cache_frames
    (frames of cache_block's pass whose K/V this pass attends to, relative to that pass's input).

    variant (Sec. 3.2): "block" feeds the block alone and reuses the cached K/V of the neighbour processed
    just before it; "extended" is the paper's B_i' = [B_{i-1}, B_i] with the feature cache standing in
    for B_{i+1}: the Num_C/2 frames of the not yet processed neighbour that touch the block are fed with
    it; "nocache" is B_i' = [B_{i-1}, B_i, B_{i+1}] fed whole, nothing cached."""
    if first_block_frames is None:
        first_block_frames = num_b
    half = num_c // 2
    assert half <= num_b, "the Num_C/2 context frames come from the adjacent block (Sec. 3.2), which has Num_B"
    frames = [first_block_frames] + [num_b] * (block_num - 1)
    starts = [0]
    for n in frames[:-1]:
        starts.append(starts[-1] + n)
    ctx = lambda b: min(half, frames[b - 1])       # frames of block b that a neighbour sees
    out = []
    for step in range(1, T + block_num):            # steps 1 .. T + Block_num - 1
        # block b entered at step b at level T and has level T - (step - b) now
        in_queue = [b for b in range(1, block_num + 1) if 1 <= T - (step - b) <= T]
        rev = order == "reverse"
        seq = sorted(in_queue, reverse=rev)          # reverse: tail (largest b) first
        prev, prev_keep = 0, 0
        for b in seq:
            level = T - (step - b)
            # the neighbours on either side count only while they are in the queue themselves
            before = ctx(b - 1) if b - 1 in in_queue else 0
            after = ctx(b + 1) if b + 1 in in_queue else 0
            if variant == "block":
                lead, trail = 0, 0
            elif variant == "extended":              # only the neighbour that is processed after this block
                lead, trail = (before, 0) if rev else (0, after)
            elif variant == "nocache":
                lead, trail = before, after
            else:
                raise ValueError(variant)
            if prev == 0 or half == 0 or variant == "nocache":
                cb, cf, cn = 0, 0, 0
            elif rev:                                 # neighbour is the later block: its first frames touch b
                cb, cn = prev, ctx(prev)
                cf = prev_keep
            else:                                     # neighbour is the earlier block: its last frames touch b
                cb, cn = prev, ctx(prev)
                cf = prev_keep + frames[prev - 1] - cn
            out.append(dict(step=step, block=b, level=level, timestep=t_max * level / T,
                            frame0=starts[b - 1], n_frames=frames[b - 1],
                            in_frame0=starts[b - 1] - lead, in_frames=lead + frames[b - 1] + trail, keep_first=lead,
                            cache_block=cb, cache_first=cf, cache_frames=cn))
            prev, prev_keep = b, lead
    return out


def bubble_ratio_reverse(N, T, block_num):
    """Eq. 3 (N <= Block_num) and Eq. 4 (N > Block_num), tail-to-head order, as printed."""
    if N <= block_num:
        bubble = N * N - N - 1
    else:
        bubble = block_num * (N - T) + N * (T - 2) + 1
    return bubble / (bubble + T * block_num)


def bubble_ratio_sequential(N, T, block_num):
    """Eq. 5, head-to-tail order, as printed."""
    bubble = N * N - 1
    return bubble / (bubble + T * block_num)
