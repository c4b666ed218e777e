"""ess_decode_step on seeded random configurations against the oracle: shapes, formats, schedules, pool sizes and
ragged context lengths drawn together, so that combinations no hand-written case has are met too.  Indices, miss
counts and cache state must be identical; attention within the 2e-2 contract (the tighter gates of the other tests
hold for all but lists of a handful of quantised entries, where a head's few bf16-rounded weights do not average out)."""
import random

import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _qbits, _topk_sets_equal

pytestmark = pytest.mark.gpu


def _draw(case):
    rnd = random.Random(7000 + case)
    T = rnd.choice([1, 1, 2])
    B = rnd.randint(1, 5)
    Hi = rnd.choice([16, 24, 32, 48, 64])
    Di = rnd.choice([32, 64, 128])
    k = rnd.choice([16, 64, 128, 256, 512, 1024, 2048])
    L = max(2 * k * T, 300) + rnd.choice([100, 1000, 5000, 12000])
    L = (rnd.randint(max(2 * k * T, 300), L) + 63) // 64 * 64
    H = rnd.choice([8, 16, 40, 64, 128])
    fmt = rnd.choice([0, 0, 1])
    flags = rnd.choice([0, 1, 2, 4, 4]) | rnd.choice([0, 0, 16])
    offload = rnd.random() < 0.8
    S = rnd.randint(T * k, L) if offload else L
    rho = rnd.choice([0.3, 0.7, 0.9])
    lens = [rnd.randint(T, L) for _ in range(B)]
    if rnd.random() < 0.5:
        lens[0] = L
    thr = rnd.choice([0, 50, 400])
    return dict(B=B, T=T, Hi=Hi, Di=Di, k=k, L=L, H=H, fmt=fmt, flags=flags, S=S, offload=offload, rho=rho, lens=lens, thr=thr)


@pytest.mark.parametrize("case", range(24))
def test_decode_step_random_configuration(ess_lib, case):
    from paper_2512_10576_amd import binding as bnd
    c = _draw(case)
    print("random configuration", case, c, flush=True)
    B, T, Hi, Di, k, L, H, fmt, S = (c[x] for x in ("B", "T", "Hi", "Di", "k", "L", "H", "fmt", "S"))
    stride = 1152 if fmt == 0 else 656
    sd = 7000 + case
    qi, w, key = synth.indexer_inputs(sd, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor(c["lens"], dtype=torch.int32)
    host = (synth.latent_rows_bf16(sd, B * L) if fmt == 0 else synth.latent_rows_fp8(sd, B * L)).reshape(B, L, stride)
    sets = None
    if c["offload"]:
        try:                                     # the trace generator needs k positions to draw from in every row
            trace = synth.TopkTrace(sd, ctx_len, T, k, c["rho"])
            sets = [trace.next() for _ in range(3)]
        except RuntimeError:
            sets = None
    ctx = bnd.Context(bnd.make_config(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
                                      slots_per_seq=S, flags=c["flags"], latent_fmt=fmt, row_stride=stride))
    poison = 0x7F if fmt == 0 else 0x7E          # never-filled slots must not be read
    oc = O.SlotCache(B, L, S)
    if c["offload"]:
        hp = torch.empty((B, L, stride), dtype=torch.uint8, pin_memory=True)
        hp.copy_(host)
        cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp, slot_pool=torch.full((B, S, stride), poison, dtype=torch.uint8, device="cuda"))
        opool = np.full((B, S, stride), poison, np.uint8)
    else:
        cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=host.clone().cuda())
        opool = host.numpy().copy()
        oc.make_resident_identity()
    ctx.cache_reset(cache, B)
    if c["flags"] & 4:
        ctx.set_overlap_threshold(c["thr"])
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    mc = torch.empty((B,), dtype=torch.int32, device="cuda")
    dev = [x.cuda() for x in (qi, w, key, ctx_len)]
    for step in range(1, 4):
        q = synth.attn_query(sd + step, B, T, H)
        ov = sets[step - 1] if (sets is not None and step != 2) else None       # step 2 uses the real top-k
        r = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx_len.numpy(), k, oc, opool, host.numpy() if c["offload"] else None,
                          _qbits(q), fmt, 576 ** -0.5, step, None if ov is None else ov.numpy())
        ctx.decode_step(cache, dev[0], dev[1], dev[2], dev[3], q.cuda(), step, idx_out, out, lse, mc, None if ov is None else ov.cuda())
        torch.cuda.synchronize()
        _topk_sets_equal(idx_out.cpu().numpy(), r["idx"])
        assert np.array_equal(mc.cpu().numpy(), r["miss_count"]), step
        if c["offload"]:                         # (nothing offloaded: the library keeps no LRU state, slot = position)
            assert np.array_equal(cache.slot_of.cpu().numpy(), oc.slot_of), step
            assert np.array_equal(cache.token_of.cpu().numpy(), oc.token_of), step
            assert np.array_equal(cache.stamp.cpu().numpy().view(np.uint32), oc.stamp), step
            assert np.array_equal(cache.slot_pool.cpu().numpy(), opool), step
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - r["out"]) <= 2e-2 + 2e-2 * np.abs(r["out"])), step
        lg = lse.cpu().numpy().astype(np.float64)
        fin = np.isfinite(r["lse"])
        assert np.array_equal(np.isneginf(lg), np.isneginf(r["lse"])), step
        assert np.allclose(lg[fin], r["lse"][fin], atol=1e-2, rtol=1e-4), step
    ctx.close()
