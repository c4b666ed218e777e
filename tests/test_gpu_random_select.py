"""Stages 1-2 on seeded random shapes with few distinct scores (small integer operands: ties by the thousand, and in
a third of the cases a run of identical keys a third of the context long), through the three selection paths --
ess_index_score + ess_topk, ess_index_topk (no score array), ess_topk_static -- against the oracle: scores and
selected sets identical."""
import random

import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _topk_sets_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", range(12))
def test_selection_paths_random_shape_with_ties(ess_lib, case):
    from paper_2512_10576_amd import binding as bnd
    rnd = random.Random(9000 + case)
    T = rnd.choice([1, 1, 2, 3, 4])
    B = rnd.randint(1, 4)
    Hi = rnd.choice([4, 16, 24, 32, 64])
    Di = rnd.choice([32, 64, 128])
    k = rnd.choice([16, 64, 256, 1024, 2048])
    L = rnd.choice([300, 2000, 9000, 20000]) + rnd.randint(0, 500)
    qk, wl = rnd.choice([1, 1, 2, 8]), rnd.choice([1, 2, 8])
    lens = [rnd.randint(T, L) for _ in range(B)]
    if rnd.random() < 0.6:
        lens[0] = L
    print("selection", case, dict(B=B, T=T, Hi=Hi, Di=Di, k=k, L=L, qk=qk, wl=wl, lens=lens), flush=True)
    q, w, key = synth.indexer_inputs(9000 + case, B, T, Hi, Di, L, qk, wl, 16)
    if rnd.random() < 0.3:
        a = rnd.randint(0, L // 2)
        key[:, a:a + L // 3] = key[:, a:a + 1]
    ctx_len = torch.tensor(lens, dtype=torch.int32)
    sc = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx_len.numpy())
    ref = O.topk(sc, ctx_len.numpy(), k)
    ctx = bnd.Context(bnd.make_config(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=8))
    d = [x.cuda() for x in (q, w, key, ctx_len)]
    score = torch.empty((B, T, L), dtype=torch.float32, device="cuda")
    idx = torch.full((B, T, k), -7, dtype=torch.int32, device="cuda")
    ctx.index_score(d[0], d[1], d[2], d[3], score)
    ctx.topk(score, d[3], idx)
    torch.cuda.synchronize()
    got = score.cpu().numpy()
    for b in range(B):
        for t in range(T):
            vis = max(0, lens[b] - (T - 1 - t))
            assert np.array_equal(got[b, t, :vis], sc[b, t, :vis].astype(np.float32)), (b, t)
    _topk_sets_equal(idx.cpu().numpy(), ref)
    idx.fill_(-7)
    ctx.index_topk(d[0], d[1], d[2], d[3], idx)
    torch.cuda.synchronize()
    _topk_sets_equal(idx.cpu().numpy(), ref)
    idx.fill_(-7)
    bnd.topk_static(score, d[3], idx)
    torch.cuda.synchronize()
    _topk_sets_equal(idx.cpu().numpy(), ref)
    ctx.close()
