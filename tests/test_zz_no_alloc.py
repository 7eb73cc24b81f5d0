"""strp_mask_topk_static (the entry point that allocates nothing) against strp_mask_topk on the same scores."""
import numpy as np
import pytest
import torch

from paper_2510_03246_amd import strp

pytestmark = pytest.mark.gpu


def _scores(n, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    s = torch.randn(n, generator=g, device="cuda") ** 2
    s[torch.randint(0, n, (n // 50,), generator=g, device="cuda")] = float(s[0].item())     # ties, some at the threshold
    return s


def test_static_topk_matches_the_workspace_variant_on_two_calls_in_a_row():
    """First 48 x 28672 scores (the multi-block path, all of the static scratch's levels in use), then a smaller input
    straight after it on the same array (which still holds the first call's candidates and counters), then a vector one
    block handles, and the size limit.  mask, idx and tau are bit-equal to strp_mask_topk's."""
    ctx = strp.Context(0)
    ref_ctx = strp.Context(0)
    n_max = 48 * 28672
    mask = torch.empty(n_max, dtype=torch.uint8, device="cuda")
    idx = torch.empty(n_max, dtype=torch.int32, device="cuda")
    tau = torch.empty(1, dtype=torch.float32, device="cuda")
    cases = [(n_max, int(0.3 * n_max), 1), (200003, 120000, 2), (28672, 8602, 3), (70001, 1, 4), (70001, 70000, 5)]
    scores = [(_scores(n, seed), k) for n, k, seed in cases]
    refs = [ref_ctx.strp_mask_topk(s, k) for s, k in scores]      # allocates its outputs and workspace: done beforehand
    torch.cuda.synchronize()

    def allocations():   # allocation requests served by torch's caching allocator so far (frees do not lower it)
        return torch.cuda.memory_stats().get("allocation.all.allocated", 0)

    for (s, k), (mask_r, idx_r, tau_r) in zip(scores, refs):
        n = s.numel()
        mask.fill_(7)
        idx.fill_(-1)
        before = allocations()
        ctx.strp_mask_topk_static(s, k, mask, idx, tau)
        assert allocations() == before
        torch.cuda.synchronize()
        assert torch.equal(mask[:n], mask_r), n
        assert torch.equal(idx[:k], idx_r), n
        assert bool((idx[k:] == -1).all()) and bool((mask[n:] == 7).all())
        assert float(tau.item()) == float(tau_r.item())
    assert ctx.ws is None                                        # the static variant never needed a workspace
    with pytest.raises(strp.StrpError) as e:
        big = torch.zeros(1, dtype=torch.float32, device="cuda")
        ctx.check(ctx.lib.strp_mask_topk_static(ctx.h, big.data_ptr(), 1572864 + 1, 5, mask.data_ptr(), idx.data_ptr(),
                                                tau.data_ptr()))
    assert e.value.status == strp.EINVAL
    ctx.close()
    ref_ctx.close()
