"""The index build that allocates nothing (cf_build_keep_index_static) against the ordinary entry
point: bit-exact idx, cu_kept and N_k on two calls in a row, the second on a smaller input, through
the C ABI with caller-owned buffers only."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2502_00340_amd import binding as Bn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(mask_np, idx, cu, n_dev):
    B, S = mask_np.shape
    mask = torch.from_numpy(mask_np).to(DEV)
    ridx, rcu, rn_dev, rn = Bn.build_keep_index(mask)          # the existing entry point (workspace argument)
    idx.fill_(-7)
    cu.fill_(-7)
    n_dev.fill_(-7)
    lib = Bn.lib()
    vp = lambda t: C.c_void_p(t.data_ptr())
    rc = lib.cf_build_keep_index_static(vp(mask), B, S, vp(idx), vp(cu), vp(n_dev),
                                        C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, rc
    torch.cuda.synchronize()
    n = int(n_dev.item())
    assert n == rn == int(mask_np.astype(bool).sum())
    assert torch.equal(cu[:B + 1], rcu)
    assert torch.equal(idx[:n], ridx[:n])
    assert np.array_equal(idx[:n].cpu().numpy(), np.flatnonzero(mask_np.reshape(-1)).astype(np.int32))
    return n


def test_static_scratch_index_build_matches_the_workspace_one_on_two_calls_in_a_row():
    print("[case] no-alloc keep index, two calls", flush=True)
    rng = np.random.default_rng(11)
    # caller-owned buffers, sized once for the larger call
    idx = torch.empty(3 * 40961, dtype=torch.int32, device=DEV)
    cu = torch.empty(8, dtype=torch.int32, device=DEV)
    n_dev = torch.empty(1, dtype=torch.int32, device=DEV)
    big = (rng.random((3, 40961)) < 0.5).astype(np.uint8)       # 31 blocks: the per-block counts go through the scratch
    small = (rng.random((2, 20000)) < 0.3).astype(np.uint8)     # 10 blocks: a shorter prefix of the same scratch
    n1 = _both(big, idx, cu, n_dev)
    n2 = _both(small, idx, cu, n_dev)
    assert n1 > n2 > 0
    tiny = (rng.random((2, 300)) < 0.5).astype(np.uint8)        # one block: no scratch at all
    _both(tiny, idx, cu, n_dev)


def test_static_scratch_index_build_at_its_maximum_size():
    print("[case] no-alloc keep index, 2^24 tokens", flush=True)
    rng = np.random.default_rng(12)
    mask = (rng.random((4, 1 << 22)) < 0.5).astype(np.uint8)
    idx = torch.empty(1 << 24, dtype=torch.int32, device=DEV)
    cu = torch.empty(5, dtype=torch.int32, device=DEV)
    n_dev = torch.empty(1, dtype=torch.int32, device=DEV)
    _both(mask, idx, cu, n_dev)
