"""Oracle of the block-wise denoising queue and the bubble-ratio closed forms (TEST INFRASTRUCTURE).

Queue (paper Sec. 3.1): the video is cut into Block_num temporal blocks; one new
block enters the FIFO queue's tail at the highest noise level at each diffusion
step, every block in the queue is processed once per step from tail (noisiest)
to head (cleanest), every processed block drops one noise level, and the head
leaves the queue once it is clean.  Feature cache (Sec. 3.2): a block reuses the
self-attention K/V of the block processed immediately before it in the same
step.  First block is longer by Num_C/2 frames (Sec. 3.3).
"""


def blockwise_schedule(T, block_num, num_b, num_c, first_block_frames=None, t_max=1000.0, order="reverse"):
    """List of block passes in execution order.  Each pass is a dict:
    step (1-based diffusion step), block (1-based, video order), level (T..1), timestep,
    frame0, n_frames, cache_block (0 = none), cache_first, cache_frames (frames of cache_block's
    K/V this pass attends to, relative to that block's first frame)."""
    if first_block_frames is None:
        first_block_frames = num_b
    half = num_c // 2
    frames = [first_block_frames] + [num_b] * (block_num - 1)
    starts = [0]
    for n in frames[:-1]:
        starts.append(starts[-1] + n)
    out = []
    for step in range(1, T + block_num):            # steps 1 .. T + Block_num - 1
        # block b entered at step b at level T and has level T - (step - b) now
        in_queue = [b for b in range(1, block_num + 1) if 1 <= T - (step - b) <= T]
        seq = sorted(in_queue, reverse=(order == "reverse"))     # reverse: tail (largest b) first
        prev = 0
        for b in seq:
            level = T - (step - b)
            if prev == 0 or half == 0:
                cb, cf, cn = 0, 0, 0
            elif order == "reverse":                  # neighbour is the later block: its first frames touch b
                cb, cf, cn = prev, 0, min(half, frames[prev - 1])
            else:                                     # neighbour is the earlier block: its last frames touch b
                cn = min(half, frames[prev - 1])
                cb, cf = prev, frames[prev - 1] - cn
            out.append(dict(step=step, block=b, level=level, timestep=t_max * level / T,
                            frame0=starts[b - 1], n_frames=frames[b - 1],
                            cache_block=cb, cache_first=cf, cache_frames=cn))
            prev = b
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
