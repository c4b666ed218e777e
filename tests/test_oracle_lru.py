"""Pins for the oracle's Sparse Memory Pool bookkeeping (CPU only): a trace
worked by hand, a textbook LRU in the one-access-per-step special case, and
invariants on random traces."""
import os
from collections import OrderedDict

import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_trace():
    c = O.SlotCache(1, 16, 4)
    for line in open(os.path.join(GOLD, "lru_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        step, sel, miss, vict, tok, stamp = [[int(x) for x in f.split()] for f in line.split("|")]
        idx = np.full((1, 1, 4), -1, np.int32)
        idx[0, 0, : len(sel)] = sel
        r = c.step(idx, step[0])
        assert r["miss_tok"][0].tolist() == miss
        assert r["victims"][0].tolist() == vict
        assert c.token_of[0].tolist() == tok
        assert c.stamp[0].tolist() == stamp
        assert r["miss_count"][0] == len(miss)
        assert r["slot_idx"][0, 0, : len(sel)].tolist() == [tok.index(s) for s in sel]
        assert r["fresh"][0, 0, : len(sel)].tolist() == [s in miss for s in sel]


def test_one_access_per_step_is_textbook_lru():
    rng = np.random.default_rng(2)
    L, S = 40, 6
    c = O.SlotCache(1, L, S)
    lru = OrderedDict()
    for step in range(1, 400):
        s = int(rng.zipf(1.3) % L)
        r = c.step(np.array([[[s]]], np.int32), step)
        hit = s in lru
        if hit:
            lru.move_to_end(s)
        else:
            if len(lru) == S:
                lru.popitem(last=False)
            lru[s] = True
        assert (r["miss_count"][0] == 0) == hit
        assert set(c.token_of[0][c.token_of[0] >= 0].tolist()) == set(lru.keys())


def _check_state(c):
    for b in range(c.B):
        res = np.nonzero(c.slot_of[b] >= 0)[0]
        assert len(res) <= c.S
        assert np.array_equal(c.token_of[b, c.slot_of[b, res]], res)
        occ = np.nonzero(c.token_of[b] >= 0)[0]
        assert np.array_equal(c.slot_of[b, c.token_of[b, occ]], occ)
        assert len(occ) == len(res)


def test_random_trace_invariants_and_lossless_rows():
    B, L, S, T, k = 3, 300, 64, 2, 24
    rng = np.random.default_rng(7)
    host = rng.integers(0, 256, size=(B, L, 16), dtype=np.uint8)
    pool = np.full((B, S, 16), 0xEE, np.uint8)
    c = O.SlotCache(B, L, S)
    for step in range(1, 30):
        idx = np.stack([np.stack([rng.choice(L, k, replace=False) for _ in range(T)]) for _ in range(B)]).astype(np.int32)
        idx[0, 0, -3:] = -1
        before = c.slot_of.copy()
        r = c.step(idx, step)
        O.fill_slots(pool, host, r["miss_tok"], r["victims"])
        _check_state(c)
        for b in range(B):
            R = np.unique(idx[b][idx[b] >= 0])
            assert np.all(c.slot_of[b, R] >= 0)                        # everything selected is resident
            was = before[b, R] >= 0
            assert np.array_equal(c.slot_of[b, R[was]], before[b, R[was]])   # hits are never moved
            assert r["miss_count"][b] == (~was).sum()
            assert np.all(c.stamp[b, c.slot_of[b, R]] == step)
            occ = np.nonzero(c.token_of[b] >= 0)[0]
            assert np.array_equal(pool[b, occ], host[b, c.token_of[b, occ]])  # slot bytes == host bytes
            rows = O.gather_rows(pool, r["slot_idx"])
            v = idx[b] >= 0
            assert np.array_equal(rows[b][v], host[b, idx[b][v]])
            assert not rows[b][~v].any()


def test_full_ratio_never_misses_twice_and_overlap_bounds_misses():
    B, L, k = 2, 2048, 64
    ctx = torch.full((B,), L, dtype=torch.int32)
    tr = synth.TopkTrace(3, ctx, 1, k, 0.75)
    full = O.SlotCache(B, L, L)
    small = O.SlotCache(B, L, 4 * k)
    seen = [set(), set()]
    for step in range(1, 12):
        idx = tr.next().numpy()
        rf = full.step(idx, step)
        rs = small.step(idx, step)
        for b in range(B):
            new = set(idx[b, 0].tolist()) - seen[b]
            assert rf["miss_count"][b] == len(new)
            seen[b] |= set(idx[b, 0].tolist())
            if step > 1:
                assert rs["miss_count"][b] <= k - int(0.75 * k)


def test_capacity_error_and_identity_mode():
    c = O.SlotCache(1, 32, 4)
    with pytest.raises(ValueError):
        c.step(np.arange(5, dtype=np.int32).reshape(1, 1, 5), 1)
    d = O.SlotCache(1, 8, 8)
    d.make_resident_identity()
    r = d.step(np.array([[[7, 0, 3]]], np.int32), 1)
    assert r["miss_count"][0] == 0 and r["slot_idx"].tolist() == [[[7, 0, 3]]]
