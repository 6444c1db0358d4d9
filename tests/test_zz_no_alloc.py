"""GPU test of the allocation-free entry point moe_permute_noalloc (scratch in a fixed device
array inside the library) against moe_permute (scratch in the caller's workspace) and against the
oracle's grouping: bit-exact, on two calls in a row, the second with a smaller input, so that what
the first call left in the shared scratch array must not matter."""
import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
from oracle import moe_oracle as mo
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _outputs(cfg):
    P = cfg.T * cfg.K
    return (torch.full((cfg.E,), -1, dtype=torch.int32, device=gu.DEV),
            torch.full((cfg.E + 1,), -1, dtype=torch.int32, device=gu.DEV),
            torch.full((P,), -1, dtype=torch.int32, device=gu.DEV),
            torch.full((P,), -1, dtype=torch.int32, device=gu.DEV))


def test_permute_noalloc_equals_permute_on_two_calls_in_a_row():
    gen = torch.Generator(device="cpu").manual_seed(7)
    for T, E, K in ((40000, 128, 8), (3001, 37, 5)):          # 157 segments of 2048 ids, then 8
        print(f"case noalloc T={T} E={E} K={K}", flush=True)
        cfg = moe.make_config(T, 256, E, K, 256, moe.DTYPE_BF16, moe.DTYPE_BF16)
        # skewed expert ids (squares of uniforms), as routing produces them
        idx_h = (torch.rand((T, K), generator=gen) ** 2 * E).to(torch.int32).clamp_(0, E - 1)
        idx = idx_h.to(gu.DEV)
        want = moe.moe_permute(cfg, idx)[:4]
        out = _outputs(cfg)
        torch.cuda.synchronize()
        # number of allocation requests torch's allocator has served so far (a count of events: it
        # cannot fall when the garbage collector frees tensors of earlier tests in between)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        moe.moe_permute_noalloc(cfg, idx, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        for got, ref in zip(out, want):
            assert torch.equal(got, ref)
        counts, offsets, perm, inv = mo.group_by_expert(idx_h.numpy(), E)
        assert np.array_equal(out[0].cpu().numpy(), counts) and np.array_equal(out[1].cpu().numpy(), offsets)
        assert np.array_equal(out[2].cpu().numpy(), perm) and np.array_equal(out[3].cpu().numpy(), inv)


def test_permute_noalloc_rejects_what_does_not_fit():
    cfg = moe.make_config(1 << 20, 256, 1024, 2, 256, moe.DTYPE_BF16, moe.DTYPE_BF16)    # 1024 segments x 1024 experts x 4 B = 4 MiB
    assert moe.moe_workspace_bytes(cfg, moe.CALL_PERMUTE) > (1 << 20)
    idx = torch.zeros((8, 2), dtype=torch.int32, device=gu.DEV)         # never read: the size check comes first
    out = tuple(torch.zeros(8, dtype=torch.int32, device=gu.DEV) for _ in range(4))
    with pytest.raises(moe.MoEError) as e:
        moe.moe_permute_noalloc(cfg, idx, out)
    assert e.value.status == -8
    assert all(int(o.sum()) == 0 for o in out)
    torch.cuda.synchronize()
