"""Pins for the oracle's append (CPU only): a trace worked by hand, a textbook
LRU when every step appends one token and selects one, and a decode loop over
an appended context against the same loop over a context built whole."""
import os
from collections import OrderedDict

import numpy as np
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_append_trace():
    S, L, Di, R = 3, 10, 4, 16
    rng = np.random.default_rng(0)
    c = O.SlotCache(1, L, S)
    key = np.zeros((1, L, Di), np.uint8)
    host = rng.integers(1, 255, size=(1, L, R), dtype=np.uint8)
    pool = np.zeros((1, S, R), np.uint8)
    ctx_len = np.array([4], np.int32)
    n_app = 0
    for line in open(os.path.join(GOLD, "append_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        op, step = f[0].split()[0], int(f[0].split()[1])
        tok, stamp, clen = [int(x) for x in f[3].split()], [int(x) for x in f[4].split()], int(f[5])
        if op == "sel":
            sel = [int(x) for x in f[1].split()]
            idx = np.array(sel, np.int32).reshape(1, 1, -1)
            r = c.step(idx, step)
            O.fill_slots(pool, host, r["miss_tok"], r["victims"])
        else:
            n_app += 1
            nk = np.full((1, 1, Di), 100 + n_app, np.uint8)
            nr = np.full((1, 1, R), 200 + n_app, np.uint8)
            before = int(ctx_len[0])
            placed = O.append_tokens(c, key, host, pool, ctx_len, nk, nr, step)
            assert placed.tolist() == [[int(f[2])]]
            if before < L:                               # written to both caches at its position
                assert (key[0, before] == 100 + n_app).all() and (host[0, before] == 200 + n_app).all()
        assert c.token_of[0].tolist() == tok, line
        assert c.stamp[0].tolist() == stamp, line
        assert int(ctx_len[0]) == clen, line
        occ = np.nonzero(c.token_of[0] >= 0)[0]
        assert np.array_equal(pool[0, occ], host[0, c.token_of[0, occ]])     # a slot holds its token's bytes
        assert np.array_equal(c.slot_of[0, c.token_of[0, occ]], occ)


def test_append_plus_one_selection_per_step_is_textbook_lru():
    """each step touches one old token, then appends one: the resident set must follow an OrderedDict LRU"""
    rng = np.random.default_rng(5)
    L, S, R = 300, 7, 8
    c = O.SlotCache(1, L, S)
    key = np.zeros((1, L, 4), np.uint8)
    host = rng.integers(0, 256, size=(1, L, R), dtype=np.uint8)
    pool = np.zeros((1, S, R), np.uint8)
    ctx_len = np.array([20], np.int32)
    lru = OrderedDict()

    def touch(tok):
        if tok in lru:
            lru.move_to_end(tok)
        else:
            if len(lru) == S:
                lru.popitem(last=False)
            lru[tok] = True

    step = 0
    while ctx_len[0] < L:
        step += 1
        s = int(ctx_len[0]) - 1 - (int(rng.zipf(1.2)) - 1) % int(ctx_len[0])
        r = c.step(np.array([[[s]]], np.int32), step)                 # one selection: stamp `step`
        O.fill_slots(pool, host, r["miss_tok"], r["victims"])
        touch(s)
        step += 1                                                     # the append gets a step number of its own
        p = int(ctx_len[0])
        placed = O.append_tokens(c, key, host, pool, ctx_len, np.zeros((1, 1, 4), np.uint8),
                                 rng.integers(0, 256, size=(1, 1, R), dtype=np.uint8), step)
        touch(p)
        assert placed[0, 0] >= 0 and ctx_len[0] == p + 1
        assert set(c.token_of[0][c.token_of[0] >= 0].tolist()) == set(lru.keys())
        occ = np.nonzero(c.token_of[0] >= 0)[0]
        assert np.array_equal(pool[0, occ], host[0, c.token_of[0, occ]])


def _bits(q):
    return q.view(torch.int16).numpy().view(np.uint16)


def test_decode_over_appended_context_equals_context_built_whole():
    """Grow the caches token by token with append_tokens, run decode steps in between, and compare every
    step with a decode over caches that were built in one piece with the same content (offloaded and fully
    resident): pins positions, the ctx_len update and that appended bytes land where the path reads them."""
    B, T, Hi, Di, Lmax, k, H, S = 2, 2, 4, 32, 96, 8, 4, 40
    L0 = np.array([30, 41], np.int32)
    steps = 6
    qi, w, key_all = synth.indexer_inputs(3, B, T, Hi, Di, Lmax, 4, 4, 8)
    qi, w, key_all = qi.numpy(), w.numpy(), key_all.numpy()
    rows_all = synth.latent_rows_bf16(3, B * Lmax).reshape(B, Lmax, 1152).numpy()
    for offloaded in (True, False):
        Sx = S if offloaded else Lmax
        # grown state: only the first L0 tokens exist at the start
        key_g = np.zeros_like(key_all); host_g = np.zeros_like(rows_all)
        for b in range(B):
            key_g[b, : L0[b]] = key_all[b, : L0[b]]
            host_g[b, : L0[b]] = rows_all[b, : L0[b]]
        cg = O.SlotCache(B, Lmax, Sx)
        pool_g = np.zeros((B, Sx, 1152), np.uint8)
        if not offloaded:
            cg.make_resident_identity()
            pool_g[:] = host_g
        ctx_g = L0.copy()
        for step in range(1, steps + 1):
            q = synth.attn_query(10 + step, B, T, H)
            rg = O.decode_step(qi, w, key_g, ctx_g, k, cg, pool_g, host_g if offloaded else None, _bits(q), 0,
                               576 ** -0.5, step)
            # whole-built reference: all content present, fresh cold pool, same visible length
            cw = O.SlotCache(B, Lmax, Lmax); cw.make_resident_identity()
            rw = O.decode_step(qi, w, key_all, ctx_g, k, cw, rows_all.copy(), None, _bits(q), 0, 576 ** -0.5, step)
            assert np.array_equal(rg["idx"], rw["idx"])
            np.testing.assert_allclose(rg["out"], rw["out"], rtol=0, atol=1e-12)
            np.testing.assert_allclose(rg["lse"], rw["lse"], rtol=0, atol=1e-12)
            new_key = np.stack([key_all[b, ctx_g[b]: ctx_g[b] + T] for b in range(B)])
            new_rows = np.stack([rows_all[b, ctx_g[b]: ctx_g[b] + T] for b in range(B)])
            before = ctx_g.copy()
            placed = O.append_tokens(cg, key_g, host_g if offloaded else None, pool_g, ctx_g, new_key, new_rows, step)
            assert np.array_equal(ctx_g, before + T)
            assert (placed >= 0).all()
            for b in range(B):
                assert np.array_equal(key_g[b, : ctx_g[b]], key_all[b, : ctx_g[b]])
                if offloaded:
                    assert np.array_equal(host_g[b, : ctx_g[b]], rows_all[b, : ctx_g[b]])
                    assert not host_g[b, ctx_g[b]:].any()
                assert not key_g[b, ctx_g[b]:].any()
                occ = np.nonzero(cg.token_of[b] >= 0)[0]
                if offloaded:
                    assert np.array_equal(pool_g[b, occ], rows_all[b, cg.token_of[b, occ]])
                    assert np.all(cg.stamp[b, cg.slot_of[b, before[b]: ctx_g[b]]] == step)


def test_append_at_the_end_of_the_buffer_drops_and_saturates():
    B, T, L, S = 1, 2, 6, 4
    c = O.SlotCache(B, L, S)
    key = np.zeros((B, L, 4), np.uint8); host = np.zeros((B, L, 8), np.uint8); pool = np.zeros((B, S, 8), np.uint8)
    ctx_len = np.array([5], np.int32)
    placed = O.append_tokens(c, key, host, pool, ctx_len, np.full((B, T, 4), 9, np.uint8), np.full((B, T, 8), 7, np.uint8), 1)
    assert ctx_len[0] == 6 and placed[0, 0] >= 0 and placed[0, 1] == -1
    assert (key[0, 5] == 9).all() and (host[0, 5] == 7).all()
    placed = O.append_tokens(c, key, host, pool, ctx_len, np.full((B, T, 4), 1, np.uint8), np.full((B, T, 8), 1, np.uint8), 2)
    assert ctx_len[0] == 6 and (placed == -1).all() and (key[0, 5] == 9).all()
