"""spion_pattern_static, the entry point that allocates nothing and takes no workspace (its scratch is
an array inside the library's device image), against spion_pattern on the same inputs: every output
bit-exact, on two calls in a row that share the scratch, the second on a smaller problem."""
import numpy as np
import pytest
import torch

import spion_inputs as si

pytestmark = pytest.mark.gpu


def _outputs(nb, dev):
    i32 = dict(dtype=torch.int32, device=dev)
    return dict(fl_out=torch.full((nb, nb), 255, dtype=torch.uint8, device=dev),
                row_ptr=torch.full((nb + 1,), -7, **i32), col_idx=torch.full((nb * nb,), -7, **i32),
                col_ptr=torch.full((nb + 1,), -7, **i32), row_idx=torch.full((nb * nb,), -7, **i32),
                bsr_pos=torch.full((nb * nb,), -7, **i32), nnzb=torch.full((1,), -7, **i32),
                pool_sum=torch.full((nb, nb), -7, dtype=torch.int64, device=dev))


def _map(L, seed):
    rng = np.random.default_rng(seed)
    A = (rng.random((L, L), dtype=np.float32) ** 6).astype(np.float32)
    A[:, L // 3:L // 3 + 8] += 0.4
    i = np.arange(L)
    A[i, i] += 0.3
    return np.minimum(A, 1.0).astype(np.float32)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import paper_2309_12578_amd as sp
    sp.load()
    dev = torch.device("cuda:0")
    # two calls in a row on the shared scratch: a large block grid first (nb = 128, cell arrays beyond
    # LDS), then a smaller problem (nb = 24) whose scratch region still holds the first call's values;
    # then the largest grid the entry point accepts, with pool_sum left to the scratch (NULL output)
    cases = [(2048, 16, 3, si.T_QUANTILE, 0.95, 0, True), (768, 32, 31, si.T_MEAN_KSTD, 0.5, 0, True),
             (4096, 16, 5, si.T_QUANTILE, 0.98, sp.SPION_PATTERN_NO_FILL, False)]
    for k, (L, block, filt, mode, value, flags, with_pool) in enumerate(cases):
        nb = L // block
        A = torch.from_numpy(_map(L, 40 + k)).to(dev)
        want, got = _outputs(nb, dev), _outputs(nb, dev)
        ws = torch.empty(sp.spion_pattern_workspace_bytes(L, block), dtype=torch.uint8, device=dev)
        sp.spion_pattern(A, L, block, filt, mode, value, want["fl_out"], want["row_ptr"], want["col_idx"],
                         want["col_ptr"], want["row_idx"], want["bsr_pos"], want["nnzb"],
                         want["pool_sum"] if with_pool else None, ws, flags=flags)
        sp.spion_pattern_static(A, L, block, filt, mode, value, got["fl_out"], got["row_ptr"], got["col_idx"],
                                got["col_ptr"], got["row_idx"], got["bsr_pos"], got["nnzb"],
                                got["pool_sum"] if with_pool else None, flags=flags)
        torch.cuda.synchronize()
        n = int(want["nnzb"].item())
        assert 0 < n < nb * nb and int(got["nnzb"].item()) == n
        for name in ("fl_out", "row_ptr", "col_ptr", "pool_sum"):
            assert torch.equal(got[name], want[name]), (k, name)
        for name in ("col_idx", "row_idx", "bsr_pos"):
            assert torch.equal(got[name][:n], want[name][:n]), (k, name)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2309_12578_amd as sp
    sp.load()
    dev = torch.device("cuda:0")
    L, block = 8192, 16                       # nb = 512 > SPION_STATIC_MAX_NB
    nb = L // block
    A = torch.zeros((64, 64), device=dev)     # never read: the call is refused on the host
    out = _outputs(4, dev)
    with pytest.raises(sp.SpionError) as e:
        sp.spion_pattern_static(A, L, block, 3, si.T_QUANTILE, 0.9, out["fl_out"], out["row_ptr"],
                                out["col_idx"], out["col_ptr"], out["row_idx"], out["bsr_pos"], out["nnzb"], None)
    assert e.value.code == -8 and "scratch" in str(e.value)
    assert nb > 256 and int(out["nnzb"].item()) == -7          # nothing was enqueued
