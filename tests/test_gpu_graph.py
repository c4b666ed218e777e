"""A resident decode step captured in a HIP graph: every replay is checked against the CPU oracle, with
new inputs copied into the captured buffers and ordinary eager work between the replays.  (An offloaded
step carries the step number, the LRU time stamp, as a launch argument, so a captured one would
repeat its stamp: callers update that argument or launch those steps eagerly.)"""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _check_attn, _ctx, _qbits, _topk_sets_equal

pytestmark = pytest.mark.gpu


def test_resident_decode_step_replayed_from_a_graph(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    print("graph capture of a resident decode step", flush=True)
    B, T, Hi, Di, L, k, H = 2, 2, 64, 128, 5000, 512, 128
    ctx_len = torch.tensor([5000, 3777], dtype=torch.int32)
    pool = synth.latent_rows_bf16(3, B * L).reshape(B, L, 1152)
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H)
    cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=pool.cuda())
    ctx.cache_reset(cache, B)
    qi0, w0, key = synth.indexer_inputs(10, B, T, Hi, Di, L, 8, 8, 16)
    dqi, dw, dkey, dlen = qi0.cuda(), w0.cuda(), key.cuda(), ctx_len.cuda()
    dq = synth.attn_query(10, B, T, H).cuda()
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    mc = torch.full((B,), 7, dtype=torch.int32, device="cuda")

    def reference(qi, w, q):
        oc = O.SlotCache(B, L, L)
        oc.make_resident_identity()
        return O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx_len.numpy(), k, oc, pool.numpy().copy(), None,
                             _qbits(q), O.FMT_BF16, 576 ** -0.5, 1)

    # eager run first (also the warm-up the capture needs)
    ctx.decode_step(cache, dqi, dw, dkey, dlen, dq, 1, idx_out, out, lse, mc)
    torch.cuda.synchronize()
    r = reference(qi0, w0, dq.cpu())
    _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
    _check_attn(out, lse, r["out"], r["lse"])

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctx.decode_step(cache, dqi, dw, dkey, dlen, dq, 1, idx_out, out, lse, mc)
    for rep in range(3):
        print("  replay", rep, flush=True)
        qi, w, _ = synth.indexer_inputs(20 + rep, B, T, Hi, Di, 64, 8, 8, 16)      # new queries, same keys
        q = synth.attn_query(20 + rep, B, T, H)
        dqi.copy_(qi); dw.copy_(w); dq.copy_(q)
        out.zero_(); idx_out.zero_(); mc.fill_(9)                                   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        r = reference(qi, w, q)
        _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
        _check_attn(out, lse, r["out"], r["lse"])
        assert mc.cpu().tolist() == [0, 0]
    ctx.close()
