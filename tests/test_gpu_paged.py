"""GPU parity of the paged Indexer-Cache (ess_index_score_paged, ess_decode_step with a block table,
paged ess_append) against the CPU oracle.  Scores are compared bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _check_attn, _ctx, _qbits, _topk_sets_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,B,T,Hi,Di,Lmax,lens,pow2", [
    ("ragged64x128", 3, 1, 64, 128, 5056, [5056, 4097, 1], False),
    ("mtp2", 2, 2, 64, 128, 3008, [3008, 2051], False),
    ("heads40_d64", 2, 1, 40, 64, 768, [768, 300], False),
    ("tiny_d32", 1, 2, 4, 32, 64, [17], True),
    ("long", 2, 1, 64, 128, 40960, [40960, 33000], False),
])
def test_index_score_paged_bit_exact(ess_lib, name, B, T, Hi, Di, Lmax, lens, pow2):
    print("index_score_paged", name, flush=True)
    q, w, key = synth.indexer_inputs(200 + B, B, T, Hi, Di, Lmax, 8, 8, 16)
    ctx_len = torch.tensor(lens, dtype=torch.int32)
    pages, table, _ = synth.paged_indexer_cache(30 + B, key, ctx_len, n_spare_pages=5, pow2=pow2)
    ref = O.index_score_paged(q.numpy(), w.numpy(), pages.numpy(), table.numpy(), ctx_len.numpy())
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=Lmax, idx_heads=Hi, idx_dim=Di, topk=8, attn_heads=8)
    score = torch.full((B, T, Lmax), -7.0, dtype=torch.float32, device="cuda")
    ctx.index_score_paged(q.cuda(), w.cuda(), pages.cuda(), table.cuda(), ctx_len.cuda(), score)
    torch.cuda.synchronize()
    got = score.cpu().numpy()
    for b in range(B):
        for t in range(T):
            vis = max(lens[b] - (T - 1 - t), 0)
            assert np.array_equal(got[b, t, :vis].view(np.uint32), ref[b, t, :vis].view(np.uint32)), (b, t)
    ctx.close()


def test_decode_loop_paged_with_append(ess_lib):
    """offloaded entries, T = 2, paged index keys with scales, the context grows across a page boundary"""
    from paper_2512_10576_amd import binding as bnd
    print("paged decode loop", flush=True)
    B, T, Hi, Di, L, k, H, S = 3, 2, 64, 128, 6016, 512, 128, 1500
    qi, w, key = synth.indexer_inputs(71, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor([5040, 4349, 6013], dtype=torch.int32)
    # pages are mapped ahead of the context: up to ctx_len + 16 tokens (the last sequence runs out of pages
    # at the end of the buffer)
    pages, table, _ = synth.paged_indexer_cache(31, key, torch.clamp(ctx_len + 16, max=L), n_spare_pages=4)
    host = synth.latent_rows_bf16(71, B * L).reshape(B, L, 1152)
    hp = torch.empty((B, L, 1152), dtype=torch.uint8, pin_memory=True); hp.copy_(host)
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
               slots_per_seq=S)
    cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
    ctx.cache_reset(cache, B)
    oc = O.SlotCache(B, L, S)
    opool = np.zeros((B, S, 1152), np.uint8)
    opages, otable, ohost, octx = pages.numpy().copy(), table.numpy(), host.numpy().copy(), ctx_len.numpy().copy()
    dpages, dtable, dctx = pages.cuda(), table.cuda(), ctx_len.cuda()
    dqi, dw = qi.cuda(), w.cuda()
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    placed = torch.empty((B, T), dtype=torch.int32, device="cuda")
    g = torch.Generator().manual_seed(5)
    for step in range(1, 11):
        q = synth.attn_query(70 + step, B, T, H)
        r = O.decode_step(qi.numpy(), w.numpy(), None, octx, k, oc, opool, ohost, _qbits(q), 0, 576 ** -0.5, step,
                          paged=(opages, otable))
        ctx.decode_step(cache, dqi, dw, dpages, dctx, q.cuda(), step, idx_out, out, lse, block_table=dtable)
        _, _, nk = synth.indexer_inputs(300 + step, B, 1, Hi, Di, T, 8, 8, 16)
        nr = synth.latent_rows_bf16(300 + step, B * T).reshape(B, T, 1152)
        ns = (0.25 + torch.rand((B, T), generator=g)).to(torch.float32)
        ref_placed = O.append_tokens(oc, None, ohost, opool, octx, nk.numpy(), nr.numpy(), step,
                                     paged=(opages, otable, ns.numpy()))
        ctx.append(cache, nk.contiguous().cuda(), nr.contiguous().cuda(), dpages, dctx, step, placed, ns.cuda(), dtable)
        torch.cuda.synchronize()
        _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
        _check_attn(out, lse, r["out"], r["lse"])
        assert np.array_equal(placed.cpu().numpy(), ref_placed)
        assert np.array_equal(dctx.cpu().numpy(), octx)
        assert np.array_equal(dpages.cpu().numpy(), opages)
        assert np.array_equal(hp.numpy(), ohost)
        assert np.array_equal(cache.slot_of.cpu().numpy(), oc.slot_of)
        assert np.array_equal(cache.slot_pool.cpu().numpy(), opool)
    # the first ran out of mapped pages, the second crossed a page boundary (4352), the third hit the buffer end
    assert octx.tolist() == [5056, 4369, 6016]
    ctx.close()


def test_paged_keys_under_the_switch_with_confined_fetches(ess_lib):
    """Paged index keys in the split-batch schedule with a confined fetch (the paged index-score kernel then
    takes its work by ticket): bit-identical to the DA schedule, which the loop test above holds against
    the oracle."""
    from paper_2512_10576_amd import binding as bnd
    print("paged keys, switch with confinement", flush=True)
    B, T, Hi, Di, L, k, H, S = 6, 2, 64, 128, 6016, 512, 128, 1500
    qi, w, key = synth.indexer_inputs(73, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor([5040, 4349, 6013, 64, 3000, 6016], dtype=torch.int32)
    pages, table, _ = synth.paged_indexer_cache(33, key, ctx_len, n_spare_pages=4)
    host = synth.latent_rows_bf16(73, B * L).reshape(B, L, 1152)
    hp = torch.empty((B, L, 1152), dtype=torch.uint8, pin_memory=True); hp.copy_(host)
    qws = [tuple(x.cuda() for x in synth.indexer_inputs(73 + s, B, T, Hi, Di, L, 8, 8, 16)[:2]) for s in range(3)]
    dpages, dtable, dctx = pages.cuda(), table.cuda(), ctx_len.cuda()
    results, confined = {}, []
    for flags in (0, 4):
        ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
                   slots_per_seq=S, flags=flags)
        if flags == 4:
            ctx.set_overlap_threshold(0)
        cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
        ctx.cache_reset(cache, B)
        idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
        out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
        steps = []
        for step in range(1, 4):
            q = synth.attn_query(80 + step, B, T, H)
            ctx.decode_step(cache, qws[step - 1][0], qws[step - 1][1], dpages, dctx, q.cuda(), step, idx_out, out, lse,
                            block_table=dtable)
            torch.cuda.synchronize()
            if flags == 4:
                confined.append((ctx.last_overlap(), ctx.last_confined()))
            steps.append((idx_out.clone(), out.clone(), lse.clone(), cache.slot_of.clone()))
        assert ctx.get_stats()["steps"] == 3
        ctx.close()
        results[flags] = steps
    for s0, s4 in zip(results[0], results[4]):
        for x, y in zip(s0, s4):
            assert torch.equal(x, y)
    assert confined[0] == (0, 0) and all(m == 1 and c >= 1 for m, c in confined[1:]), confined


def test_paged_argument_errors(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    ctx = _ctx(ess_lib, max_batch=1, max_q_tokens=1, max_ctx=100, idx_heads=4, idx_dim=32, topk=8, attn_heads=8)
    q = torch.zeros((1, 1, 4, 32), dtype=torch.uint8, device="cuda")
    w = torch.zeros((1, 1, 4), dtype=torch.float32, device="cuda")
    pages = torch.zeros((2, 64 * 36), dtype=torch.uint8, device="cuda")
    table = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    cl = torch.zeros((1,), dtype=torch.int32, device="cuda")
    score = torch.zeros((1, 1, 100), dtype=torch.float32, device="cuda")
    with pytest.raises(bnd.EssError) as e:
        ctx.index_score_paged(q, w, pages, table, cl, score)        # max_ctx not a multiple of the page size
    assert e.value.code == bnd.ESS_ERR_UNSUPPORTED
    ctx.close()
