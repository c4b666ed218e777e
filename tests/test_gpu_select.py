"""GPU parity of the fused selection (index score + top-k without a score array: ess_index_topk, and stages 1-2 of
ess_decode_step) against the oracle's top-k of the oracle's scores, bit for bit.

The adversarial score rows of the stand-alone top-k tests (all equal, strictly monotone, a huge tie at the cut,
negatives and signed zeros, NaN / infinities, a huge dynamic range, short rows, 128K rows with ties at the cut) are
reproduced THROUGH the indexer: keys and queries are crafted so that the exact score of position s is a chosen
integer (two heads read base-16 digits of the positive part, two heads with negative weights those of the negative
part; every product and sum is exact in float32), and the paged form's per-key scale injects NaN, infinities and
forty orders of magnitude.  Such rows defeat the sampled lower bound (no bound, or far too many candidates), so
they also cover the path that recomputes a row from all its scores."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _ctx, _topk_sets_equal

pytestmark = pytest.mark.gpu

_DEC = O.decode_e4m3(np.arange(256, dtype=np.uint8))


def _code(v):
    """the E4M3 byte of an exactly representable value"""
    c = np.nonzero(_DEC == float(v))[0]
    assert c.size >= 1, v
    return np.uint8(c[0])


_DIGIT = np.array([_code(d) for d in range(16)], dtype=np.uint8)


def _craft(values, unit=1.0, Di=32):
    """values: int64 [B, L], |v| < 2^24.  Returns q [B,1,4,Di], w [B,1,4], key [B,L,Di] (E4M3 bytes / float32) with
    sum_j w_j max(0, q_j . key_s) == unit * values[b, s] exactly (unit a power of two)."""
    values = np.asarray(values, dtype=np.int64)
    B, L = values.shape
    assert np.abs(values).max() < 1 << 24
    pos, neg = np.maximum(values, 0), np.maximum(-values, 0)
    key = np.zeros((B, L, Di), np.uint8)
    for part, d0 in ((pos, 0), (neg, 6)):
        for i in range(6):
            key[:, :, d0 + i] = _DIGIT[(part >> (4 * i)) & 15]
    q = np.zeros((B, 1, 4, Di), np.uint8)
    place = [_code(1), _code(16), _code(256)]
    for head, d0 in ((0, 0), (1, 3), (2, 6), (3, 9)):
        for i in range(3):
            q[:, 0, head, d0 + i] = place[i]
    w = np.tile(np.array([1.0, 4096.0, -1.0, -4096.0], np.float32) * np.float32(unit), (B, 1, 1))
    return q, w, key


def _run_index_topk(ess_lib, q, w, key, lens, k, block_table=None, n_tok=None):
    q, w, key = (torch.as_tensor(x) for x in (q, w, key))
    B, T, Hi, Di = q.shape
    Lmax = key.shape[1] if block_table is None else 64 * block_table.shape[1]
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=Lmax, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=8)
    idx = torch.full((B, T, k), -5, dtype=torch.int32, device="cuda")
    bt = None if block_table is None else torch.as_tensor(block_table).cuda()
    ctx.index_topk(q.cuda(), w.cuda(), key.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), idx, block_table=bt)
    torch.cuda.synchronize()
    first = idx.cpu().numpy()
    idx.fill_(-5)                                  # a second call finds the row counters as a first one does
    ctx.index_topk(q.cuda(), w.cuda(), key.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), idx, block_table=bt)
    torch.cuda.synchronize()
    assert np.array_equal(first, idx.cpu().numpy())
    ctx.close()
    return first


def _run_decode_step(ess_lib, q, w, key, lens, k, block_table=None, flags=None):
    """stages 1-2 through ess_decode_step (fused form unless flags say otherwise), nothing offloaded (slot =
    position); returns idx_out"""
    from paper_2512_10576_amd import binding as bnd
    if flags is None:
        flags = bnd.ESS_FLAG_FUSED_SELECT
    q, w, key = (torch.as_tensor(x) for x in (q, w, key))
    B, T, Hi, Di = q.shape
    H = 8
    Lmax = key.shape[1] if block_table is None else 64 * block_table.shape[1]
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=Lmax, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H, flags=flags)
    pool = torch.zeros((B, Lmax, 1152), dtype=torch.uint8, device="cuda")
    cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=pool)
    ctx.cache_reset(cache, B)
    idx = torch.full((B, T, k), -5, dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    qa = torch.zeros((B, T, H, 576), dtype=torch.bfloat16, device="cuda")
    bt = None if block_table is None else torch.as_tensor(block_table).cuda()
    for step in (1, 2):
        ctx.decode_step(cache, q.cuda(), w.cuda(), key.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), qa, step, idx, out,
                        block_table=bt)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    ctx.close()
    return got


# ---------------------------------------------------------------- benchmark-like inputs
@pytest.mark.parametrize("name,B,T,Hi,Di,Lmax,qk,wl,wd,lens,k", [
    ("cfg1", 1, 1, 4, 32, 4096, 4, 4, 8, [4096], 256),
    ("ragged64x128", 3, 1, 64, 128, 20011, 8, 8, 16, [20011, 9000, 2050], 2048),
    ("mtp2", 2, 2, 64, 128, 20000, 8, 8, 16, [20000, 12051], 2048),
    ("heads40_d64", 2, 1, 40, 64, 9777, 8, 8, 16, [9777, 8300], 512),
    ("tiny", 1, 2, 4, 32, 40, 4, 4, 8, [17], 8),
    ("mtp3", 2, 3, 64, 128, 12000, 8, 8, 16, [12000, 9051], 1024),
    ("mtp4_heads40", 2, 4, 40, 64, 9777, 8, 8, 16, [9777, 300], 256),
    ("long", 2, 1, 64, 128, 131072, 8, 8, 16, [131072, 98304 + 12345], 2048),
])
def test_index_topk_matches_oracle(ess_lib, name, B, T, Hi, Di, Lmax, qk, wl, wd, lens, k):
    print("index_topk", name, flush=True)
    q, w, key = synth.indexer_inputs(300 + B + T, B, T, Hi, Di, Lmax, qk, wl, wd)
    sc = O.index_score(q.numpy(), w.numpy(), key.numpy(), np.array(lens))
    ref = O.topk(sc, np.array(lens), k)
    _topk_sets_equal(_run_index_topk(ess_lib, q, w, key, lens, k), ref)
    if name in ("ragged64x128", "mtp2", "tiny"):
        print("  through ess_decode_step, fused and through the score array", flush=True)
        from paper_2512_10576_amd import binding as bnd
        _topk_sets_equal(_run_decode_step(ess_lib, q, w, key, lens, k), ref)
        _topk_sets_equal(_run_decode_step(ess_lib, q, w, key, lens, k, flags=bnd.ESS_FLAG_DENSE_SCORES), ref)


@pytest.mark.parametrize("Di,Hi,T,Lmax,lens,k", [(128, 64, 2, 16384, [16384, 9001, 70], 1024), (32, 32, 1, 8256, [8256, 8193], 512)])
def test_index_topk_paged_matches_oracle(ess_lib, Di, Hi, T, Lmax, lens, k):
    print("index_topk paged Di", Di, "T", T, flush=True)
    B = len(lens)
    q, w, key = synth.indexer_inputs(77 + Di, B, T, Hi, Di, Lmax, 8, 8, 16)
    pages, table, _ = synth.paged_indexer_cache(5 + Di, key, torch.tensor(lens, dtype=torch.int32), n_spare_pages=3)
    sc = O.index_score_paged(q.numpy(), w.numpy(), pages.numpy(), table.numpy(), np.array(lens))
    ref = O.topk(sc, np.array(lens), k)
    _topk_sets_equal(_run_index_topk(ess_lib, q, w, pages, lens, k, block_table=table.numpy()), ref)
    _topk_sets_equal(_run_decode_step(ess_lib, q, w, pages, lens, k, block_table=table.numpy()), ref)


# ---------------------------------------------------------------- adversarial score rows through the indexer
def _adversarial_values(L, rng):
    rows = []
    rows.append(np.full(L, 56, np.int64))                                              # all equal
    rows.append(np.arange(L, 0, -1, dtype=np.int64))                                  # strictly decreasing
    rows.append(np.arange(L, dtype=np.int64))                                         # strictly increasing
    tie = np.zeros(L, np.int64); tie[::7] = 32; tie[5::1000] = 144                    # a huge tie at the cut
    rows.append(tie)
    rows.append(rng.integers(-3, 4, L).astype(np.int64))                              # negatives, zeros, many ties
    rows.append(np.rint(rng.normal(40000, 7000, L)).clip(0).astype(np.int64))         # the ordinary case, ties at the cut
    return np.stack(rows)


@pytest.mark.parametrize("L,k", [(40000, 2048), (131072, 2048)])
def test_selection_adversarial_rows(ess_lib, L, k):
    print("fused selection, adversarial rows of", L, flush=True)
    rng = np.random.default_rng(L)
    vals = _adversarial_values(L, rng)
    q, w, key = _craft(vals, unit=1.0 / 16)
    lens = [L, L - 3, L, min(L, 70001), L, 16385]
    sc = O.index_score(q, w, key, np.array(lens))
    assert np.array_equal(sc[0, 0, :L], (vals[0] / 16).astype(np.float32))           # the crafting does what it says
    assert np.array_equal(sc[4, 0, :L], (vals[4] / 16).astype(np.float32))
    ref = O.topk(sc, np.array(lens), k)
    _topk_sets_equal(_run_index_topk(ess_lib, q, w, key, lens, k), ref)
    _topk_sets_equal(_run_decode_step(ess_lib, q, w, key, lens, k), ref)
    print("  short rows", flush=True)
    lens2 = [100, 2048, 2049, 0, 1, 8193]
    ref2 = O.topk(O.index_score(q, w, key, np.array(lens2)), np.array(lens2), k)
    _topk_sets_equal(_run_index_topk(ess_lib, q, w, key, lens2, k), ref2)
    _topk_sets_equal(_run_decode_step(ess_lib, q, w, key, lens2, k), ref2)


def test_selection_nan_inf_and_wide_range_through_key_scales(ess_lib):
    """paged Indexer-Cache: the score is scale_s * sum; scales of +inf, NaN and 10^-20 .. 10^20 turn integer sums into
    NaN (inf * 0, NaN * x), +-inf and a huge dynamic range"""
    print("fused selection, NaN / inf / wide range", flush=True)
    L, k = 40000, 2048
    rng = np.random.default_rng(9)
    vals = np.stack([rng.integers(-3, 4, L), rng.integers(-2000, 2000, L), rng.integers(0, 3, L)]).astype(np.int64)
    q, w, key = _craft(vals)
    B = vals.shape[0]
    lens = [L, L - 1, 30001]
    pages, table, _ = synth.paged_indexer_cache(3, torch.from_numpy(key), torch.tensor(lens, dtype=torch.int32), n_spare_pages=2)
    pages = pages.numpy().copy()
    n_pages = pages.shape[0]
    pages = pages.reshape(n_pages, -1)
    flat = np.ones(n_pages * 64, np.float32)                                            # one scale per key of the pool
    pick = rng.permutation(flat.size)
    flat[pick[:300]] = np.inf
    flat[pick[300:600]] = np.nan
    wide = pick[600:flat.size // 2]
    flat[wide] = (10.0 ** rng.integers(-20, 21, wide.size)).astype(np.float32)
    pages[:, 64 * 32:] = flat.reshape(n_pages, 64).view(np.uint8)
    pages = torch.from_numpy(pages)
    sc = O.index_score_paged(q, w, pages.numpy(), table.numpy(), np.array(lens))
    vis = sc[0, 0, :L]
    assert np.isnan(vis).any() and np.isposinf(vis).any() and np.isneginf(vis).any()
    ref = O.topk(sc, np.array(lens), k)
    _topk_sets_equal(_run_index_topk(ess_lib, q, w, pages, lens, k, block_table=table.numpy()), ref)
    _topk_sets_equal(_run_decode_step(ess_lib, q, w, pages, lens, k, block_table=table.numpy()), ref)
