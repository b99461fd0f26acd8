"""GPU parity of the strided attention pattern (Sec. 3.3) with the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2408_11746_amd as mst
from oracle import attention_mask as oam

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("L,l", [(1, 1), (16, 4), (64, 3), (128, 1), (96, 7), (48, 16), (64, 100), (37, 5), (255, 16), (256, 256), (513, 128),
                                 (1024, 128), (1024, 256)])
def test_mask_equals_oracle(L, l):
    dev = torch.device("cuda:0")
    M = torch.full((L * L + 16,), 7, dtype=torch.uint8, device=dev)
    mst.mst_strided_attention_mask(M, L, l)
    torch.cuda.synchronize()
    got = M.cpu().numpy()
    assert (got[L * L:] == 7).all()                                  # nothing written past the end
    np.testing.assert_array_equal(got[:L * L].reshape(L, L), oam.strided_mask(L, l))
    assert int(got[:L * L].sum(dtype=np.int64)) == mst.mst_strided_attention_count(L, l)


def test_large_mask_properties():
    # at a size the oracle's loops do not finish: the count, sampled rows and causality
    L, l = 8192, 256
    dev = torch.device("cuda:0")
    M = torch.empty((L, L), dtype=torch.uint8, device=dev)
    mst.mst_strided_attention_mask(M, L, l)
    torch.cuda.synchronize()
    assert int(M.sum(dtype=torch.int64).item()) == mst.mst_strided_attention_count(L, l)
    assert int(torch.triu(M, 1).sum(dtype=torch.int64).item()) == 0
    rows = M[[0, 1, 255, 256, 257, 4095, 8191]].cpu().numpy()
    for r, i in zip(rows, [0, 1, 255, 256, 257, 4095, 8191]):
        want = sorted(set(range(max(i - l + 1, 0), i + 1)) | {j for j in range(i + 1) if (i - j) % l == 0})
        assert np.nonzero(r)[0].tolist() == want


def test_mask_rejects_bad_arguments():
    dev = torch.device("cuda:0")
    M = torch.empty(64, dtype=torch.uint8, device=dev)
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_mask(M, 0, 4)
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_mask(M, 8, 0)
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_mask(None, 8, 4)
    with pytest.raises(mst.MstError):
        mst.mst_strided_attention_mask(M, 40000, 4)
