"""The search entry point that allocates nothing (partial scores in the library's static device array)
against the entry point that takes a workspace: same scores, same choice, same copy of the winner, on two
calls in a row, the second on a smaller problem (the array keeps the first call's contents)."""
import numpy as np
import pytest

import paper_2302_06058_amd as bm

pytestmark = pytest.mark.gpu


def _mask_words(I, J, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 1 << 32, size=(I, (J + 31) // 32), dtype=np.uint64).astype(np.uint32)


def _both(I, J, N, M, K, seed):
    import torch
    from helpers import i32_dev
    rng = np.random.default_rng(seed + 1)
    B = i32_dev(_mask_words(I, J, seed).view(np.int32))
    perms = i32_dev(np.stack([rng.permutation(I) for _ in range(K)]).astype(np.int32))
    want = bm.bimask_perm_search(B, I, J, N, M, perms)
    scores = torch.full((K,), -1, dtype=torch.int32, device="cuda")
    best = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    best_perm = torch.full((I,), -1, dtype=torch.int32, device="cuda")
    before = torch.cuda.memory_allocated()
    bm.bimask_perm_search_static(B, I, J, N, M, perms, scores, best, best_perm)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for got, w in zip((scores, best, best_perm), want):
        assert torch.equal(got, w)


def test_static_scratch_search_equals_workspace_search_twice_in_a_row():
    _both(11008, 4096, 2, 4, 100, 9001)        # 84 partial sums per candidate
    _both(256, 2304, 2, 4, 7, 9002)            # smaller: fewer partial sums, the rest of the array is stale
    _both(64, 100, 1, 4, 150, 9003)
    _both(136, 1032, 4, 8, 13, 9004)


def test_static_scratch_limit_is_an_error_not_a_launch():
    import torch
    I, J, K = 8, 1 << 22, 100                  # 4096 column slices x 100 candidates x 4 bytes > 1 MiB
    assert bm.workspace_bytes(bm.WS_PERM_SEARCH, I, J, 0, K, bm.BF16, 2, 4) > (1 << 20)
    z = torch.zeros((16,), dtype=torch.int32, device="cuda")
    st = bm.lib().bimask_perm_search_static(z.data_ptr(), I, J, 2, 4, z.data_ptr(), K, z.data_ptr(), z.data_ptr(), None, None)
    assert st == 6
