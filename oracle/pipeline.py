"""Oracle: slot-level simulation of the device pipeline that runs the block queue (TEST INFRASTRUCTURE).

Model (paper Sec. 3.1, 3.4 and the appendix on denoising order): the DiT is split over N devices;
a block pass visits devices 1..N in order and occupies each for one slot; a device works on one pass
at a time and takes passes in the queue schedule's order; a block's pass at diffusion step s+1 can
enter device 1 only after its pass at step s has left device N (the scheduler update needs the
whole model's output).  The pass that hands the feature cache over is the one just before in the
same step, so in-order execution already satisfies it.  Idle slots of a device between its first
and its last busy slot, plus the slots it waits before its first pass and after its last one while
the job is still running elsewhere, are bubbles.

The count is independent of the paper's closed forms (Eq. 3, 4, 5).  For T > N and at least two
blocks it turns out equal to the numerators of Eq. 5 and Eq. 4 and, for tail-to-head order with
N <= Block_num, to (N-1)^2, the value Eq. 4 takes at Block_num = N, rather than the N^2-N-1 that
Eq. 3 prints; the tests pin all three.
"""
from oracle.schedule import blockwise_schedule


def simulate_pipeline(n_devices, T, block_num, order="reverse"):
    """Returns dict(makespan, busy_per_device, bubble_per_device, bubble_ratio, finish) where
    bubble_per_device counts every slot in [0, makespan) a device is not working and
    bubble_ratio = bubbles / (bubbles + busy) of one device (all devices have the same busy count)."""
    sched = blockwise_schedule(T, block_num, 1, 0, order=order)
    free_at = [0] * n_devices                 # first slot each device is free again
    done = {}                                 # block -> slot after which its latest pass left the last device
    finish = []
    for e in sched:
        t = done.get(e["block"], 0)           # cannot start before the previous step's pass is complete
        for j in range(n_devices):
            start = max(t, free_at[j])
            free_at[j] = start + 1
            t = start + 1
        done[e["block"]] = t
        finish.append(t)
    makespan = max(free_at)
    busy = len(sched)
    return dict(makespan=makespan, busy_per_device=busy, bubble_per_device=makespan - busy,
                bubble_ratio=(makespan - busy) / makespan, finish=finish)
