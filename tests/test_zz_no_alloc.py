"""The routing call that allocates nothing (realb_route_stats_static: the per-block partial histograms in
a file-scope device array instead of the context's workspace) against realb_route_stats, through the C ABI:
identical outputs, bit for bit, on two calls in a row, the second with a smaller input (the array keeps the
first call's partials, none of which the second may pick up), for both top-k kernels; and its limits."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("E,k,D", [(64, 6, 8), (128, 8, 8), (40, 4, 5), (512, 16, 8)])
def test_static_scratch_route_stats_matches_the_context_call(E, k, D):
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    print(f"[no-alloc] E={E} k={k} D={D}", flush=True)
    rng = np.random.default_rng(E + k)
    T_big, T_small = 40000, 777
    logits = rng.standard_normal((T_big, E)).astype(np.float32)
    logits[::5] = np.round(logits[::5] * 2) / 2                       # exact ties
    isv = (rng.random(T_big) < 0.7).astype(np.uint8)
    rcfg = default_config(T_big, E, k, D, 128, 128)
    ctx = R.Context(rcfg)
    lg, iv = torch.from_numpy(logits).cuda(), torch.from_numpy(isv).cuda()
    names = ("topk_ids", "topk_w", "expert_cnt", "expert_vis", "rank_load", "rank_vis")
    for T in (T_big, T_small):                                        # two calls in a row, the second smaller
        ref, got = R.LayerBuffers(rcfg, T), R.LayerBuffers(rcfg, T)
        for n in names:
            getattr(got, n).fill_(-3)
        ctx.route_stats(lg[:T], iv[:T], ref)
        R.route_stats_static(lg[:T], iv[:T], E, k, D, got)
        torch.cuda.synchronize()
        for n in names:
            a, b = getattr(ref, n), getattr(got, n)
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), (n, T)
        assert int(got.expert_cnt.sum()) == T * k and int(got.rank_load.sum()) == T * k
    # T = 0 defines the counts
    e = R.LayerBuffers(rcfg, 0)
    e.expert_cnt.fill_(5); e.rank_load.fill_(5)
    R.route_stats_static(lg[:0], iv[:0], E, k, D, e)
    torch.cuda.synchronize()
    assert not e.expert_cnt.any() and not e.rank_load.any()
    ctx.close()


def test_static_scratch_route_stats_rejects_sizes_beyond_its_array():
    import paper_2604_19503_amd as R
    from paper_2604_19503_amd.binding import default_config
    rcfg = default_config(16, 64, 2, 8, 128, 128)
    b = R.LayerBuffers(rcfg, 16)
    lg = torch.zeros((16, 1024), dtype=torch.float32, device="cuda")
    iv = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(R.RealbError, match="exceeds the static scratch"):
        R.route_stats_static(lg, iv, 1024, 2, 8, b)
    with pytest.raises(R.RealbError):
        R.route_stats_static(lg, iv, 64, 17, 8, b)
    with pytest.raises(R.RealbError):
        R.route_stats_static(lg, iv, 64, 2, 7, b)
    torch.cuda.synchronize()
