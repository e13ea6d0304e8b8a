"""GPU parity of the coordinated noise initialisation (Sec. 3.3): the library's assignment + device gather
against the oracle's, bit for bit, on the same pool and the same random words."""
import numpy as np
import pytest
import torch

from oracle.noise import gather_frames, noise_assignment
from paper_2505_21070_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,block_num,num_b,num_c,seed", [
    ("tiny", 5, 2, 2, 0),             # fp32 frames of 64 x 128
    ("small_bf16", 4, 3, 4, 1),       # bf16 frames of 72 x 256
    ("wan1p3b_stage", 8, 4, 4, 2),    # the queue workload's shape: 6 pool frames of 1560 x 1536 bf16
])
def test_blocks_from_the_pool_match_oracle(name, block_num, num_b, num_c, seed):
    from paper_2505_21070_amd import binding as B
    cfg = synth.stage_config(name)
    gen = torch.Generator().manual_seed(seed)
    pool = synth.noise_pool(cfg, num_b + num_c // 2, gen)                  # fp32 values representable in cfg dtype
    words = synth.shuffle_words((block_num - 1) * (num_b - 1), seed + 100)
    got_idx = B.noise_assign(block_num, num_b, num_c, words)
    ref_idx = noise_assignment(block_num, num_b, num_c, words)
    assert got_idx == ref_idx
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    pool_dev = pool.to(device="cuda", dtype=td).contiguous()
    pool_np = pool.numpy()
    for b, idx in enumerate(got_idx):
        out = B.noise_gather(pool_dev, torch.tensor(idx, dtype=torch.int32, device="cuda"))
        ref = gather_frames(pool_np, ref_idx[b])
        assert out.shape == ref.shape
        assert np.array_equal(out.float().cpu().numpy(), ref), f"block {b + 1}"
    # the properties the section states, on what the device produced
    half = num_c // 2
    for b in range(1, block_num):
        assert not set(got_idx[b - 1][len(got_idx[b - 1]) - half:]) & set(got_idx[b])


def test_gather_edge_cases():
    from paper_2505_21070_amd import binding as B
    pool = torch.arange(3 * 40, dtype=torch.float32, device="cuda").reshape(3, 40) + 1.0   # 160-byte frames
    idx = torch.tensor([2, 2, 0, 7, -1], dtype=torch.int32, device="cuda")                 # 7, -1: out of range
    out = B.noise_gather(pool, idx)
    want = torch.stack([pool[2], pool[2], pool[0], torch.zeros(40, device="cuda"), torch.zeros(40, device="cuda")])
    assert torch.equal(out, want)
    empty = B.noise_gather(pool, torch.zeros(0, dtype=torch.int32, device="cuda"))
    assert empty.shape == (0, 40)
    with pytest.raises(B.DualParalError) as ei:                                           # 12-byte frames
        B.noise_gather(torch.zeros((2, 3), dtype=torch.float32, device="cuda"), idx[:1])
    assert ei.value.code == B.DP_EINVAL
    torch.cuda.synchronize()
