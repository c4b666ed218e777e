"""Pins for the oracle's index score and top-k (CPU only): int64 brute force,
library matmul in a special case, invariants, exhaustive sort, adversarial ties."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth


def _ints(u8):
    return torch.as_tensor(u8).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.int64)


def _brute_score(q_u8, w, key_u8, ctx_len, den):
    """Triple loop in int64 with weights scaled to integers: score*den exactly."""
    q, key = _ints(q_u8), _ints(key_u8)
    W = np.rint(np.asarray(w, dtype=np.float64) * den).astype(np.int64)
    B, T, Hi, Di = q.shape
    Lmax = key.shape[1]
    out = np.full((B, T, Lmax), None, dtype=object)
    for b in range(B):
        for t in range(T):
            vis = int(ctx_len[b]) - (T - 1 - t)
            for s in range(max(vis, 0)):
                acc = 0
                for j in range(Hi):
                    dot = 0
                    for d in range(Di):
                        dot += int(q[b, t, j, d]) * int(key[b, s, d])
                    if dot > 0:
                        acc += int(W[b, t, j]) * dot
                out[b, t, s] = acc
    return out


@pytest.mark.parametrize("T", [1, 2])
def test_index_score_int64_brute_force(T):
    B, Hi, Di, Lmax = 2, 4, 8, 37
    q, w, key = synth.indexer_inputs(11 + T, B, T, Hi, Di, Lmax, 4, 4, 8)
    w = w * torch.tensor([1.0, -1.0, 1.0, 1.0])         # a negative weight: ReLU must act before w
    ctx = np.array([37, 20], dtype=np.int32)
    got = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx)
    ref = _brute_score(q.numpy(), w.numpy(), key.numpy(), ctx, 8)
    for b in range(B):
        for t in range(T):
            vis = ctx[b] - (T - 1 - t)
            assert np.all(np.isneginf(got[b, t, vis:]))
            assert np.array_equal(got[b, t, :vis].astype(np.float64) * 8, ref[b, t, :vis].astype(np.float64))
    assert got.dtype == np.float32


def test_index_score_reduces_to_matmul():
    # one head, unit weight, non-negative q and k: ReLU is the identity => plain matrix product
    B, T, Hi, Di, Lmax = 1, 1, 1, 32, 64
    g = torch.Generator().manual_seed(0)
    qi = torch.randint(0, 5, (B, T, Hi, Di), generator=g).float()
    ki = torch.randint(0, 5, (B, Lmax, Di), generator=g).float()
    q = qi.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    key = ki.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = O.index_score(q, np.ones((B, T, Hi), np.float32), key, np.array([Lmax]))
    ref = np.matmul(ki.numpy()[0], qi.numpy()[0, 0, 0])
    assert np.array_equal(got[0, 0], ref)


def test_index_score_invariants():
    B, T, Hi, Di, Lmax = 2, 1, 8, 16, 50
    q, w, key = synth.indexer_inputs(5, B, T, Hi, Di, Lmax, 8, 8, 16)
    ctx = np.array([50, 50])
    s0 = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx)
    assert np.all(s0 >= 0) and np.array_equal(s0 * 16, np.rint(s0 * 16))
    ph = torch.randperm(Hi, generator=torch.Generator().manual_seed(1))
    pd = torch.randperm(Di, generator=torch.Generator().manual_seed(2))
    s1 = O.index_score(q[:, :, ph].numpy(), w[:, :, ph].numpy(), key.numpy(), ctx)
    s2 = O.index_score(q[..., pd].numpy(), w.numpy(), key[..., pd].numpy(), ctx)
    assert np.array_equal(s0, s1) and np.array_equal(s0, s2)
    s3 = O.index_score(q.numpy(), (-w).numpy(), key.numpy(), ctx)
    assert np.array_equal(s0, -s3)
    # full-size exactness argument: float32 BLAS gives the same bits on integer data
    qf, kf = _ints(q.numpy()).astype(np.float32), _ints(key.numpy()).astype(np.float32)
    blas = np.maximum(kf[0] @ qf[0, 0].T, 0) @ w.numpy()[0, 0]
    assert np.array_equal(blas.astype(np.float32), s0[0, 0])


def _exhaustive(row, vis, k):
    key = [(-(float(x) if x == x else -np.inf), s) for s, x in enumerate(row[:vis])]
    order = [s for _, s in sorted(key)]
    return order[:k] + [-1] * (k - min(k, vis))


def test_topk_exhaustive_sort_with_many_ties():
    rng = np.random.default_rng(4)
    B, T, Lmax, k = 3, 2, 200, 17
    score = rng.integers(0, 12, size=(B, T, Lmax)).astype(np.float32) / 16
    ctx = np.array([200, 150, 9])
    got = O.topk(score, ctx, k)
    for b in range(B):
        for t in range(T):
            vis = ctx[b] - (T - 1 - t)
            assert list(got[b, t]) == _exhaustive(score[b, t], vis, k)


def test_topk_adversarial_cases():
    L, k = 64, 8
    ctx = np.array([L])
    eq = np.full((1, 1, L), 3.5, np.float32)
    assert list(O.topk(eq, ctx, k)[0, 0]) == list(range(k))
    dec = np.arange(L, 0, -1, dtype=np.float32).reshape(1, 1, L)
    assert list(O.topk(dec, ctx, k)[0, 0]) == list(range(k))
    inc = np.arange(L, dtype=np.float32).reshape(1, 1, L)
    assert list(O.topk(inc, ctx, k)[0, 0]) == list(range(L - 1, L - 1 - k, -1))
    # k-1 clear winners, then k+1 tied at the cut: the lowest-indexed tied one is taken
    tie = np.zeros((1, 1, L), np.float32)
    winners = [60, 50, 40, 30, 20, 10, 5]
    tie[0, 0, winners] = 9.0
    tied = [3, 7, 11, 15, 19, 23, 27, 31, 35]
    tie[0, 0, tied] = 1.0
    got = O.topk(tie, ctx, k)[0, 0]
    assert sorted(got[:7]) == sorted(winners) and got[7] == 3
    # vis < k pads with -1; k == vis is a permutation of everything
    short = O.topk(inc, np.array([5]), k)[0, 0]
    assert list(short) == [4, 3, 2, 1, 0, -1, -1, -1]
    assert sorted(O.topk(inc, np.array([8]), 8)[0, 0]) == list(range(8))
    # signed zeros compare equal, NaN ranks last, negative scores are ordered correctly
    z = np.array([[-0.0, 0.0, -1.0, np.nan, -0.0, 0.5, -np.inf, -2.0]], np.float32).reshape(1, 1, 8)
    assert list(O.topk(z, np.array([8]), 8)[0, 0]) == [5, 0, 1, 4, 2, 7, 3, 6]
    assert O.topk(z, np.array([0]), 3).tolist() == [[[-1, -1, -1]]]


def test_topk_threshold_invariants():
    B, T, Hi, Di, Lmax, k = 2, 1, 4, 32, 4096, 256
    q, w, key = synth.indexer_inputs(0, B, T, Hi, Di, Lmax, 4, 4, 8)
    ctx = np.array([4096, 3000])
    score = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx)
    idx = O.topk(score, ctx, k)
    for b in range(B):
        sel = idx[b, 0]
        assert len(set(sel.tolist())) == k and sel.min() >= 0 and sel.max() < ctx[b]
        row = score[b, 0, : ctx[b]]
        thr = row[sel].min()
        uns = np.setdiff1d(np.arange(ctx[b]), sel)
        assert row[uns].max() <= thr
        at = np.nonzero(row == thr)[0]
        n_at_sel = np.isin(at, sel).sum()
        assert np.array_equal(np.sort(sel[row[sel] == thr]), at[:n_at_sel])


def test_similarity_is_eq1_and_trace_overlap_is_exact():
    assert O.intra_layer_similarity([1, 2, 3, 4], [3, 4, 5, 6]) == 0.5
    assert O.intra_layer_similarity([1, 2], [1, 2, -1, -1]) == 1.0
    ctx = torch.tensor([3000, 2500], dtype=torch.int32)
    tr = synth.TopkTrace(1, ctx, 2, 128, 0.75)
    prev = tr.next().numpy()
    for _ in range(3):
        cur = tr.next().numpy()
        for b in range(2):
            assert len(set(cur[b, 0].tolist())) == 128 and cur[b, 0].max() < ctx[b] - 1
            assert len(set(cur[b, 1].tolist())) == 128 and cur[b, 1].max() < ctx[b]
            assert O.intra_layer_similarity(prev[b, 0], cur[b, 0]) == 0.75
            assert abs(O.intra_layer_similarity(cur[b, 0], cur[b, 1]) - 115 / 128) < 1e-9
        prev = cur
    # recency skew: the median selected position lies in the newest part of the context
    assert np.median(cur[0, 0]) > 1500
