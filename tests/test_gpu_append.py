"""GPU parity of the append path (ess_append) against the CPU oracle: a decode loop whose context grows
by T tokens per step.  Every array the call writes is compared byte for byte."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _check_attn, _ctx, _qbits, _topk_sets_equal

pytestmark = pytest.mark.gpu


def _new_entries(seed, B, T, Hi, Di, fmt, qk=8):
    _, _, nk = synth.indexer_inputs(seed, B, 1, Hi, Di, T, qk, 8, 16)          # [B,T,Di] integer-valued fp8 keys
    stride = 1152 if fmt == 0 else 656
    rows = (synth.latent_rows_bf16(seed, B * T) if fmt == 0 else synth.latent_rows_fp8(seed, B * T)).reshape(B, T, stride)
    return nk.contiguous(), rows.contiguous()


@pytest.mark.parametrize("fmt,T", [(0, 2), (1, 1)])
def test_decode_loop_with_append_offloaded(ess_lib, fmt, T):
    from paper_2512_10576_amd import binding as bnd
    print("append offloaded fmt", fmt, "T", T, flush=True)
    B, Hi, Di, L, k, H, S = 3, 64, 128, 6000, 512, 128, 1500
    stride = 1152 if fmt == 0 else 656
    qi, w, key = synth.indexer_inputs(61, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor([5000, 4321, 5997], dtype=torch.int32)              # the last one reaches the end
    host = (synth.latent_rows_bf16(61, B * L) if fmt == 0 else synth.latent_rows_fp8(61, B * L)).reshape(B, L, stride)
    hp = torch.empty((B, L, stride), dtype=torch.uint8, pin_memory=True)
    hp.copy_(host)
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
               slots_per_seq=S, latent_fmt=fmt)
    cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
    ctx.cache_reset(cache, B)
    oc = O.SlotCache(B, L, S)
    opool = np.zeros((B, S, stride), np.uint8)
    okey, ohost, octx = key.numpy().copy(), host.numpy().copy(), ctx_len.numpy().copy()
    dkey, dctx = key.cuda(), ctx_len.cuda()
    dqi, dw = qi.cuda(), w.cuda()
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    placed = torch.empty((B, T), dtype=torch.int32, device="cuda")
    for step in range(1, 6):
        q = synth.attn_query(70 + step, B, T, H)
        r = O.decode_step(qi.numpy(), w.numpy(), okey, octx, k, oc, opool, ohost, _qbits(q), fmt, 576 ** -0.5, step)
        ctx.decode_step(cache, dqi, dw, dkey, dctx, q.cuda(), step, idx_out, out, lse)
        nk, nr = _new_entries(80 + step, B, T, Hi, Di, fmt)
        ref_placed = O.append_tokens(oc, okey, ohost, opool, octx, nk.numpy(), nr.numpy(), step)
        ctx.append(cache, nk.cuda(), nr.cuda(), dkey, dctx, step, placed)
        torch.cuda.synchronize()
        _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
        _check_attn(out, lse, r["out"], r["lse"])
        assert np.array_equal(placed.cpu().numpy(), ref_placed)
        assert np.array_equal(dctx.cpu().numpy(), octx)
        assert np.array_equal(dkey.cpu().numpy(), okey)
        assert np.array_equal(hp.numpy(), ohost)
        assert np.array_equal(cache.slot_of.cpu().numpy(), oc.slot_of)
        assert np.array_equal(cache.token_of.cpu().numpy(), oc.token_of)
        assert np.array_equal(cache.stamp.cpu().numpy().view(np.uint32), oc.stamp)
        assert np.array_equal(cache.slot_pool.cpu().numpy(), opool)
    assert octx.tolist()[2] == L and (ref_placed[2] == -1).all()               # the full sequence dropped its tokens
    ctx.close()


def test_decode_loop_with_append_resident(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    print("append resident", flush=True)
    B, T, Hi, Di, L, k, H = 2, 1, 4, 32, 4096, 256, 8
    qi, w, key = synth.indexer_inputs(0, B, T, Hi, Di, L, 4, 4, 8)
    ctx_len = torch.tensor([4000, 4095], dtype=torch.int32)
    rows = synth.latent_rows_bf16(5, B * L).reshape(B, L, 1152)
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H)
    cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=rows.cuda())
    ctx.cache_reset(cache, B)
    oc = O.SlotCache(B, L, L); oc.make_resident_identity()
    opool, okey, octx = rows.numpy().copy(), key.numpy().copy(), ctx_len.numpy().copy()
    dkey, dctx = key.cuda(), ctx_len.cuda()
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    placed = torch.empty((B, T), dtype=torch.int32, device="cuda")
    for step in range(1, 4):
        q = synth.attn_query(90 + step, B, T, H)
        r = O.decode_step(qi.numpy(), w.numpy(), okey, octx, k, oc, opool, None, _qbits(q), 0, 576 ** -0.5, step)
        ctx.decode_step(cache, qi.cuda(), w.cuda(), dkey, dctx, q.cuda(), step, idx_out, out, lse)
        nk, nr = _new_entries(95 + step, B, T, Hi, Di, 0, qk=4)
        ref_placed = O.append_tokens(oc, okey, None, opool, octx, nk.numpy(), nr.numpy(), step)
        ctx.append(cache, nk.cuda(), nr.cuda(), dkey, dctx, step, placed)
        torch.cuda.synchronize()
        _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
        _check_attn(out, lse, r["out"], r["lse"])
        assert np.array_equal(placed.cpu().numpy(), ref_placed)
        assert np.array_equal(dctx.cpu().numpy(), octx) and np.array_equal(dkey.cpu().numpy(), okey)
        assert np.array_equal(cache.slot_pool.cpu().numpy(), opool)
        # without a host pool the step itself keeps no stamps; the appended positions carry the step number
        st = cache.stamp.cpu().numpy().view(np.uint32)
        for b in range(B):
            for t in range(T):
                if ref_placed[b, t] >= 0:
                    assert st[b, ref_placed[b, t]] == step
        assert np.array_equal(cache.slot_of.cpu().numpy(), oc.slot_of)
    ctx.close()


def test_append_without_a_free_slot_keeps_the_entry_in_the_host_pool(ess_lib):
    """every slot was used in this step (the two queries select disjoint sets that fill the pool): the new
    entry is written to the Indexer-Cache and the host pool but not admitted"""
    from paper_2512_10576_amd import binding as bnd
    B, T, Hi, Di, L, k, H = 1, 2, 4, 32, 4096, 256, 8
    S = T * k
    qi, w, key = synth.indexer_inputs(2, B, T, Hi, Di, L, 4, 4, 8)
    ctx_len = torch.tensor([3000], dtype=torch.int32)
    host = synth.latent_rows_bf16(6, B * L).reshape(B, L, 1152)
    hp = torch.empty((B, L, 1152), dtype=torch.uint8, pin_memory=True); hp.copy_(host)
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
               slots_per_seq=S)
    cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
    ctx.cache_reset(cache, B)
    ov = torch.arange(S, dtype=torch.int32).reshape(1, T, k) * 5                # disjoint, all visible
    oc = O.SlotCache(B, L, S); opool = np.zeros((B, S, 1152), np.uint8)
    okey, ohost, octx = key.numpy().copy(), host.numpy().copy(), ctx_len.numpy().copy()
    q = synth.attn_query(3, B, T, H)
    O.decode_step(qi.numpy(), w.numpy(), okey, octx, k, oc, opool, ohost, _qbits(q), 0, 576 ** -0.5, 1, ov.numpy())
    dkey, dctx = key.cuda(), ctx_len.cuda()
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    ctx.decode_step(cache, qi.cuda(), w.cuda(), dkey, dctx, q.cuda(), 1, idx_out, out, None, None, ov.cuda())
    nk, nr = _new_entries(4, B, T, Hi, Di, 0, qk=4)
    ref_placed = O.append_tokens(oc, okey, ohost, opool, octx, nk.numpy(), nr.numpy(), 1)
    placed = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ctx.append(cache, nk.cuda(), nr.cuda(), dkey, dctx, 1, placed)
    torch.cuda.synchronize()
    assert (ref_placed == -1).all() and np.array_equal(placed.cpu().numpy(), ref_placed)
    assert dctx.item() == 3002 and np.array_equal(hp.numpy(), ohost) and np.array_equal(dkey.cpu().numpy(), okey)
    assert np.array_equal(cache.slot_of.cpu().numpy(), oc.slot_of)
    assert np.array_equal(cache.slot_pool.cpu().numpy(), opool)
    # a later step number frees the slots: the next append is admitted
    ref_placed = O.append_tokens(oc, okey, ohost, opool, octx, nk.numpy(), nr.numpy(), 2)
    ctx.append(cache, nk.cuda(), nr.cuda(), dkey, dctx, 2, placed)
    torch.cuda.synchronize()
    assert (ref_placed >= 0).all() and np.array_equal(placed.cpu().numpy(), ref_placed)
    assert np.array_equal(cache.slot_pool.cpu().numpy(), opool) and np.array_equal(cache.token_of.cpu().numpy(), oc.token_of)
    ctx.close()


def test_append_argument_errors(ess_lib):
    from paper_2512_10576_amd import binding as bnd
    ctx = _ctx(ess_lib, max_batch=2, max_q_tokens=1, max_ctx=256, idx_heads=4, idx_dim=32, topk=8, attn_heads=8)
    cache = bnd.Cache.allocate(ctx.cfg, 2)
    nk = torch.zeros((2, 1, 32), dtype=torch.uint8, device="cuda")
    nr = torch.zeros((2, 1, 1152), dtype=torch.uint8, device="cuda")
    key = torch.zeros((2, 256, 32), dtype=torch.uint8, device="cuda")
    cl = torch.zeros((2,), dtype=torch.int32, device="cuda")
    with pytest.raises(bnd.EssError):
        ctx.append(cache, nk, nr, key, cl, 0)                                   # step 0
    with pytest.raises(bnd.EssError):
        ctx.append(cache, torch.zeros((3, 1, 32), dtype=torch.uint8, device="cuda"), nr, key, cl, 1)   # B > max_batch
    ctx.close()
