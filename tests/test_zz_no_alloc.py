"""ann_score_pairs_noalloc (the entry point for callers that cannot allocate device memory) against
ann_score_pairs, through the C ABI: same kernels, so the scores must be the same bit for bit, and both within
the 16-bit bar of the oracle.  Two calls in a row share the library's one scratch array; the second is smaller."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from workloads import PRESETS, make_workload, scaled, to_host

pytestmark = pytest.mark.gpu

ann = pytest.importorskip("paper_2502_11490_amd")


def _pairs(cfg, Q, M, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randint(0, Q, (M,), generator=g, dtype=torch.int32)
    it = torch.randint(0, cfg.N, (M,), generator=g, dtype=torch.int32)
    return q.cuda(), it.cuda()


def _noalloc_raw(lib, g, m, users, q_idx, item, out):
    """The call exactly as a C caller makes it: bare pointers, no Python-side allocation."""
    return lib.ann_score_pairs_noalloc(g.handle, m.handle, users.data_ptr(), users.shape[0], q_idx.numel(),
                                       q_idx.data_ptr(), item.data_ptr(), out.data_ptr(),
                                       ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("preset,N", [("C3", 30000), ("C2", 20000), ("C4", 20000)])
def test_noalloc_matches_allocating_entry_point(preset, N):
    cfg = scaled(PRESETS[preset], N, Q=96)
    wl = make_workload(cfg, device="cuda:0", with_graph=True)
    g = ann.ann_graph_load(wl["adj"], wl["emb"])
    m = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_BF16)
    assert ann.ann_mlp_uses_mfma(m)
    lib = ann.load_library()
    h = to_host(wl)
    mlp = oracle.Mlp(h["W"], h["b"], h["head_w"])
    # first call: several batches and a ragged tail; second call: fewer queries and fewer pairs
    for Q, M, seed in ((96, 5000 + 37, 1), (17, 301, 2)):
        users = wl["users"][:Q].contiguous()
        q_idx, item = _pairs(cfg, Q, M, seed)
        want = ann.ann_score_pairs(g, m, users, q_idx, item)
        out = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda:0")
        # torch's count of allocation events only grows, whatever the garbage collector frees meanwhile
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        rc = _noalloc_raw(lib, g, m, users, q_idx, item, out)
        assert rc == 0, ann.ann_last_error()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        torch.cuda.synchronize()
        assert torch.equal(out, want), float((out - want).abs().max())
        exact = oracle.score_pairs(h["emb"], h["users"][:Q], mlp, q_idx.cpu().numpy(), item.cpu().numpy(), n_threads=8)
        assert np.max(np.abs(out.cpu().numpy() - exact)) <= 1e-2


def test_noalloc_fp32_and_limits():
    cfg = PRESETS["C1"]
    wl = make_workload(cfg, device="cuda:0")
    g = ann.ann_graph_load(wl["adj"], wl["emb"])
    m = ann.ann_mlp_load(wl["W"], wl["b"], wl["head_w"], cfg.d, ann.ANN_F32)
    q_idx, item = _pairs(cfg, cfg.Q, 777, 3)
    want = ann.ann_score_pairs(g, m, wl["users"], q_idx, item)
    out = torch.empty(777, dtype=torch.float32, device="cuda:0")
    ann.ann_score_pairs_noalloc(g, m, wl["users"], q_idx, item, out)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    # beyond the fixed array: 4,097 queries of a 512-wide first layer
    c3 = scaled(PRESETS["C3"], 5000, Q=4097)
    wl3 = make_workload(c3, device="cuda:0")
    g3 = ann.ann_graph_load(wl3["adj"], wl3["emb"])
    m3 = ann.ann_mlp_load(wl3["W"], wl3["b"], wl3["head_w"], c3.d, ann.ANN_BF16)
    q3, i3 = _pairs(c3, 4097, 64, 4)
    out3 = torch.empty(64, dtype=torch.float32, device="cuda:0")
    with pytest.raises(ann.AnnError) as e:
        ann.ann_score_pairs_noalloc(g3, m3, wl3["users"], q3, i3, out3)
    assert e.value.code == ann.binding.ANN_EINVAL and "scratch" in str(e.value)
    # exactly at the limit it runs
    users = wl3["users"][:4096].contiguous()
    q3 = q3.clamp(max=4095)
    ann.ann_score_pairs_noalloc(g3, m3, users, q3, i3, out3)
    torch.cuda.synchronize()
    assert torch.equal(out3, ann.ann_score_pairs(g3, m3, users, q3, i3))
