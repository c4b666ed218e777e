"""ess_topk_static, the entry point that allocates nothing (its scratch memory is an array inside the library's
image), against ess_topk and the CPU oracle: two calls in a row on the same GPU, the second with a smaller input,
so that what the first call left in the shared scratch array must not leak into the second."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O

pytestmark = pytest.mark.gpu


def _scores(rng, B, T, L):
    # a 1/16 grid with many ties at the cut, like the index scores of the benchmark inputs
    return (np.rint(rng.normal(40000, 7000, (B, T, L))).clip(0) / 16).astype(np.float32)


def test_topk_static_matches_topk_on_two_calls_in_a_row(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    rng = np.random.default_rng(17)
    calls = [
        # rows shared by several workgroups (long rows, few of them): the scratch lists and counters are used
        dict(B=3, T=2, L=131072, k=2048, lens=[131072, 98304 + 4321, 70000]),
        # smaller in every respect; still long enough for the shared path
        dict(B=2, T=1, L=65536, k=512, lens=[65536, 40000]),
        # a short-row call (one workgroup per row) after them
        dict(B=4, T=1, L=5000, k=256, lens=[5000, 4097, 100, 0]),
    ]
    for n, c in enumerate(calls):
        print("ess_topk_static call", n, c["B"], c["T"], c["L"], c["k"], flush=True)
        B, T, L, k = c["B"], c["T"], c["L"], c["k"]
        sc = _scores(rng, B, T, L)
        lens = np.array(c["lens"], dtype=np.int32)
        d_sc, d_len = torch.from_numpy(sc).cuda(), torch.from_numpy(lens).cuda()
        got = torch.full((B, T, k), -5, dtype=torch.int32, device="cuda")
        bnd.topk_static(d_sc, d_len, got)
        torch.cuda.synchronize()
        ctx = bnd.Context(bnd.make_config(B, T, L, 4, 32, k, 8))
        want = torch.full((B, T, k), -6, dtype=torch.int32, device="cuda")
        ctx.topk(d_sc, d_len, want)
        torch.cuda.synchronize()
        ctx.close()
        assert torch.equal(got, want)                                     # bit for bit what ess_topk gives
        ref = O.topk(sc, lens, k)
        g = got.cpu().numpy()
        for b in range(B):
            for t in range(T):
                nv = int((ref[b, t] >= 0).sum())
                assert np.array_equal(g[b, t, :nv], np.sort(ref[b, t, :nv])) and np.all(g[b, t, nv:] == -1)


def test_topk_static_rejects_sizes_beyond_its_scratch(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    sc = torch.zeros((129, 1, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(bnd.EssError) as ei:
        bnd.topk_static(sc, torch.zeros(129, dtype=torch.int32, device="cuda"),
                        torch.zeros((129, 1, 8), dtype=torch.int32, device="cuda"))
    assert ei.value.code == bnd.ESS_ERR_CAPACITY and "128" in str(ei.value)
    sc = torch.zeros((1, 1, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(bnd.EssError) as ei:
        bnd.topk_static(sc, torch.zeros(1, dtype=torch.int32, device="cuda"),
                        torch.zeros((1, 1, 4097), dtype=torch.int32, device="cuda"))
    assert ei.value.code == bnd.ESS_ERR_CAPACITY
