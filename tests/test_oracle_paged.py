"""Pins for the oracle's paged index score (CPU only): identity paging with unit scales against the flat
definition, independence from page placement, float64 brute force with the scale inside the ReLU, and
exact equality for power-of-two scales."""
import numpy as np
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth


def _inputs(seed, B, T, Hi, Di, Lmax, lens):
    q, w, key = synth.indexer_inputs(seed, B, T, Hi, Di, Lmax, 8, 8, 16)
    return q, w, key, torch.tensor(lens, dtype=torch.int32)


def test_page_layout_constants():
    assert O.PAGE_TOKENS == 64 and O.page_bytes(128) == 64 * 132
    # the paper's 16.8 %: Indexer-Cache bytes per token over all cache bytes per token (Sec. 3)
    assert abs(132 / (132 + 656) - 0.168) < 5e-4


def test_identity_paging_with_unit_scales_is_the_flat_score():
    B, T, Hi, Di, Lmax = 2, 2, 8, 32, 256
    q, w, key, ctx_len = _inputs(1, B, T, Hi, Di, Lmax, [256, 131])
    npp = Lmax // 64
    pages = np.zeros((B * npp, O.page_bytes(Di)), np.uint8)
    for b in range(B):
        for p in range(npp):
            pages[b * npp + p, : 64 * Di] = key[b, p * 64:(p + 1) * 64].numpy().reshape(-1)
            pages[b * npp + p, 64 * Di:] = np.ones(64, np.float32).view(np.uint8)
    table = np.arange(B * npp, dtype=np.int32).reshape(B, npp)
    got = O.index_score_paged(q.numpy(), w.numpy(), pages, table, ctx_len.numpy())
    ref = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx_len.numpy())
    assert np.array_equal(got, ref)


def test_page_placement_does_not_matter_and_unmapped_pages_are_never_read():
    B, T, Hi, Di, Lmax = 3, 1, 4, 32, 320
    q, w, key, ctx_len = _inputs(2, B, T, Hi, Di, Lmax, [320, 65, 7])
    a = synth.paged_indexer_cache(10, key, ctx_len, n_spare_pages=4)
    b = synth.paged_indexer_cache(11, key, ctx_len, n_spare_pages=1)
    # same scales in both poolings: copy a's scales into b's pages
    pb, tb = b[0].numpy().copy(), b[1].numpy()
    sc = a[2].numpy()
    for s_b in range(B):
        for pg in range(tb.shape[1]):
            if tb[s_b, pg] >= 0:
                pb[tb[s_b, pg], 64 * Di:] = sc[s_b, pg * 64:(pg + 1) * 64].view(np.uint8)
    ra = O.index_score_paged(q.numpy(), w.numpy(), a[0].numpy(), a[1].numpy(), ctx_len.numpy())
    rb = O.index_score_paged(q.numpy(), w.numpy(), pb, tb, ctx_len.numpy())
    assert not np.array_equal(a[1].numpy(), tb)
    assert np.array_equal(ra, rb)
    assert np.isfinite(ra[0, 0, :320]).all() and np.isneginf(ra[1, 0, 65:]).all()   # NaN spare pages never leak


def test_scale_inside_the_relu_float64_brute_force():
    B, T, Hi, Di, Lmax = 2, 2, 4, 32, 128
    q, w, key, ctx_len = _inputs(3, B, T, Hi, Di, Lmax, [128, 77])
    pages, table, scales = synth.paged_indexer_cache(12, key, ctx_len)
    got = O.index_score_paged(q.numpy(), w.numpy(), pages.numpy(), table.numpy(), ctx_len.numpy())
    tab = O.e4m3fn_table()
    qf, kf = tab[q.numpy()], tab[key.numpy()]
    for b in range(B):
        for t in range(T):
            vis = int(ctx_len[b]) - (T - 1 - t)
            for s in range(vis):
                acc = 0.0
                for j in range(Hi):
                    dot = float(np.dot(qf[b, t, j], float(scales[b, s]) * kf[b, s]))     # scaled key, as stored
                    acc += float(w[b, t, j]) * max(0.0, dot)
                assert abs(got[b, t, s] - acc) <= 1e-6 * max(abs(acc), 1e-30), (b, t, s)
            assert np.isneginf(got[b, t, vis:]).all()


def test_power_of_two_scales_are_exact():
    B, T, Hi, Di, Lmax = 1, 1, 8, 64, 192
    q, w, key, ctx_len = _inputs(4, B, T, Hi, Di, Lmax, [190])
    pages, table, scales = synth.paged_indexer_cache(13, key, ctx_len, pow2=True)
    got = O.index_score_paged(q.numpy(), w.numpy(), pages.numpy(), table.numpy(), ctx_len.numpy())
    flat = O.index_score(q.numpy(), w.numpy(), key.numpy(), ctx_len.numpy())
    assert np.array_equal(got[0, 0, :190], flat[0, 0, :190] * scales[0, :190].numpy())
    assert len(np.unique(scales.numpy())) > 3


def test_paged_append_then_score_equals_pool_built_whole():
    """append keys one page boundary across; the paged score over the grown pool equals the score over a
    pool paged from the complete flat keys with the same scales"""
    B, T, Hi, Di, Lmax = 2, 2, 4, 32, 256
    q, w, key, _ = _inputs(5, B, T, Hi, Di, Lmax, [0, 0])
    full_len = torch.tensor([200, 131], dtype=torch.int32)
    start = np.array([120, 63], np.int32)
    pages_w, table, scales = synth.paged_indexer_cache(14, key, full_len)
    pages_w, table, scales = pages_w.numpy(), table.numpy(), scales.numpy()
    # grown pool: same table, content only up to `start`
    pages_g = pages_w.copy()
    for b in range(B):
        for s in range(int(start[b]), int(full_len[b])):
            pg, r = table[b, s // 64], s % 64
            pages_g[pg, r * Di:(r + 1) * Di] = 0xFF
            pages_g[pg, 64 * Di + 4 * r: 64 * Di + 4 * r + 4] = np.float32("nan").reshape(1).view(np.uint8)
    S = 8
    c = O.SlotCache(B, Lmax, S)
    host = np.zeros((B, Lmax, 16), np.uint8); pool = np.zeros((B, S, 16), np.uint8)
    ctx_len = start.copy()
    step = 0
    while (ctx_len < full_len.numpy()).any():
        step += 1
        nk = np.stack([key[b, ctx_len[b]: ctx_len[b] + T].numpy() if ctx_len[b] + T <= Lmax else np.zeros((T, Di), np.uint8)
                       for b in range(B)])
        ns = np.stack([scales[b, ctx_len[b]: ctx_len[b] + T] for b in range(B)])
        live = ctx_len < full_len.numpy()
        before = ctx_len.copy()
        O.append_tokens(c, None, host, pool, ctx_len, nk, np.zeros((B, T, 16), np.uint8), step, paged=(pages_g, table, ns))
        ctx_len[~live] = before[~live]                      # a finished sequence stops (its extra writes are past full_len)
        ctx_len = np.minimum(ctx_len, full_len.numpy() + T)
    lens = np.minimum(ctx_len, full_len.numpy()).astype(np.int32)
    got = O.index_score_paged(q.numpy(), w.numpy(), pages_g, table, lens)
    ref = O.index_score_paged(q.numpy(), w.numpy(), pages_w, table, lens)
    assert np.array_equal(lens, full_len.numpy())
    assert np.array_equal(got, ref)


def test_paged_append_drops_tokens_whose_page_is_unmapped():
    Di = 32
    key = torch.zeros((1, 128, Di), dtype=torch.uint8)
    pages, table, _ = synth.paged_indexer_cache(15, key, torch.tensor([64], dtype=torch.int32))
    pages, table = pages.numpy(), table.numpy()
    assert table[0, 0] >= 0 and table[0, 1] == -1
    c = O.SlotCache(1, 128, 4)
    host = np.zeros((1, 128, 16), np.uint8); pool = np.zeros((1, 4, 16), np.uint8)
    ctx_len = np.array([63], np.int32)
    placed = O.append_tokens(c, None, host, pool, ctx_len, np.full((1, 2, Di), 3, np.uint8), np.full((1, 2, 16), 9, np.uint8),
                             1, paged=(pages, table, np.full((1, 2), 0.5, np.float32)))
    assert ctx_len[0] == 64 and placed[0, 0] >= 0 and placed[0, 1] == -1
    pg = pages[table[0, 0]]
    assert (pg[63 * Di: 64 * Di] == 3).all() and pg[64 * Di + 4 * 63: 64 * Di + 4 * 64].view(np.float32)[0] == 0.5
