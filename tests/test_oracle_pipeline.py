"""Pins of the pipeline simulation: hand-countable cases, conservation, and the paper's qualitative claims
about the bubble (Sec. 3.4, appendix)."""
import pytest

from oracle.pipeline import simulate_pipeline
from oracle.schedule import bubble_ratio_reverse, bubble_ratio_sequential


def test_single_device_never_idles():
    for T, B in [(1, 1), (5, 3), (8, 8)]:
        r = simulate_pipeline(1, T, B)
        assert r["makespan"] == T * B and r["bubble_per_device"] == 0


def test_single_block_is_a_plain_loop():
    # one block, N devices: every step is N slots with one device busy at a time
    r = simulate_pipeline(4, 5, 1)
    assert r["makespan"] == 4 * 5 and r["busy_per_device"] == 5 and r["bubble_per_device"] == 15


def test_two_devices_two_blocks_by_hand():
    # T = 2, tail to head.  step 1: pass a = block 1.  step 2: b = block 2, c = block 1.  step 3: d = block 2.
    # device 1: a@0, b@1, c@2 (block 1's first pass left device 2 at slot 2), d@3 (block 2's left at 3)
    # device 2: a@1, b@2, c@3, d@4  -> makespan 5, 4 busy slots each, 1 bubble each
    r = simulate_pipeline(2, 2, 2)
    assert r["finish"] == [2, 3, 4, 5] and r["makespan"] == 5 and r["bubble_per_device"] == 1


@pytest.mark.parametrize("N,T,B", [(4, 50, 4), (4, 50, 8), (8, 50, 64), (2, 8, 8), (4, 10, 3)])
def test_conservation_and_bounds(N, T, B):
    r = simulate_pipeline(N, T, B)
    assert r["busy_per_device"] == T * B
    assert r["makespan"] >= T * B + N - 1                 # at least the fill/drain of a perfect pipeline
    assert r["makespan"] <= N * T * B                     # at worst fully serial
    assert r["finish"] == sorted(r["finish"])


def test_claims_about_the_bubble():
    # the bubble ratio goes to zero as the video grows (Sec. 3.4)
    ratios = [simulate_pipeline(4, 50, B)["bubble_ratio"] for B in (4, 16, 64, 256)]
    assert ratios == sorted(ratios, reverse=True) and ratios[-1] < 0.01
    # once the queue holds at least N blocks no device idles: the bubble count stops growing with Block_num
    b = [simulate_pipeline(4, 50, B)["bubble_per_device"] for B in (8, 16, 64)]
    assert b[0] == b[1] == b[2]
    # tail-to-head order idles no more than head-to-tail (appendix)
    for N, T, B in [(4, 50, 4), (4, 50, 8), (8, 50, 16), (2, 8, 8)]:
        assert simulate_pipeline(N, T, B, "reverse")["bubble_per_device"] <= simulate_pipeline(N, T, B, "sequential")["bubble_per_device"]
    # same order of magnitude as the printed closed forms for the paper's example (5.2 % / 7.0 %)
    r = simulate_pipeline(4, 50, 4)["bubble_ratio"]
    assert 0.5 * bubble_ratio_reverse(4, 50, 4) < r < 3 * bubble_ratio_reverse(4, 50, 4)
    s = simulate_pipeline(4, 50, 4, "sequential")["bubble_ratio"]
    assert 0.5 * bubble_ratio_sequential(4, 50, 4) < s < 3 * bubble_ratio_sequential(4, 50, 4)


def test_slot_count_reproduces_the_printed_closed_forms():
    """For T > N and at least two blocks the slot count equals the numerator of Eq. 5 (head-to-tail order,
    N <= Block_num) and of Eq. 4 (tail-to-head, N > Block_num) exactly.  For tail-to-head with N <= Block_num it
    equals (N-1)^2, which is Eq. 4 evaluated at Block_num = N, and not the N^2-N-1 printed in Eq. 3."""
    for N in range(1, 9):
        for T in (N + 1, N + 2, 10, 50):
            if T <= N:
                continue
            for B in range(2, 13):
                rev = simulate_pipeline(N, T, B, "reverse")
                seq = simulate_pipeline(N, T, B, "sequential")
                if N > B:
                    eq4 = B * (N - T) + N * (T - 2) + 1
                    assert rev["bubble_per_device"] == eq4
                    assert rev["bubble_ratio"] == pytest.approx(bubble_ratio_reverse(N, T, B))
                else:
                    assert rev["bubble_per_device"] == (N - 1) ** 2
                    assert seq["bubble_per_device"] == N * N - 1
                    assert seq["bubble_ratio"] == pytest.approx(bubble_ratio_sequential(N, T, B))
    # the paper's example (N = 4, T = 50, Block_num = 4): 9 idle slots of 209, 4.3 %, against the printed 11 / 211
    r = simulate_pipeline(4, 50, 4)
    assert (r["bubble_per_device"], r["makespan"]) == (9, 209)
