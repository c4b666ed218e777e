"""GPU edge cases: empty and tiny contexts, odd sizes, maximum sizes, the non-register bookkeeping path."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth

pytestmark = pytest.mark.gpu


def _ctx(**kw):
    from paper_2512_10576_amd import binding as b
    return b.Context(b.make_config(**kw))


def _qbits(q):
    return q.view(torch.int16).cpu().numpy().view(np.uint16)


def test_decode_step_with_empty_and_tiny_contexts(ess_lib):
    """ctx_len 0, 1, 2 (T = 2: query 0 of a length-1 context sees nothing), k not a multiple of the tile"""
    from paper_2512_10576_amd import binding as bnd
    print("edges: empty / tiny contexts", flush=True)
    B, T, Hi, Di, L, k, H = 5, 2, 64, 128, 300, 100, 24
    qi, w, key = synth.indexer_inputs(61, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor([0, 1, 2, 300, 57], dtype=torch.int32)
    pool = synth.latent_rows_bf16(61, B * L).reshape(B, L, 1152)
    q = synth.attn_query(61, B, T, H)
    oc = O.SlotCache(B, L, L)
    oc.make_resident_identity()
    r = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx_len.numpy(), k, oc, pool.numpy().copy(), None,
                      _qbits(q), O.FMT_BF16, 576 ** -0.5, 1)
    ctx = _ctx(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H)
    cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=pool.cuda())
    ctx.cache_reset(cache, B)
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.full((B, T, H, 512), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, T, H), 7.0, dtype=torch.float32, device="cuda")
    ctx.decode_step(cache, qi.cuda(), w.cuda(), key.cuda(), ctx_len.cuda(), q.cuda(), 1, idx_out, out, lse)
    torch.cuda.synchronize()
    got = idx_out.cpu().numpy()
    for b in range(B):
        for t in range(T):
            ref = r["idx"][b, t]
            nv = int((ref >= 0).sum())
            assert np.array_equal(got[b, t, :nv], np.sort(ref[:nv])) and np.all(got[b, t, nv:] == -1)
    o = out.float().cpu().numpy().astype(np.float64)
    # outputs here reach O(1) (a one- or two-row selection returns the rows themselves), so the bound
    # carries the bf16 output rounding: 2^-8 relative
    assert np.all(np.abs(o - r["out"]) <= 3e-3 + 2.0 ** -8 * np.abs(r["out"]))
    lg = lse.cpu().numpy()
    assert np.array_equal(np.isneginf(lg), np.isneginf(r["lse"]))          # empty selections: lse = -inf, out = 0
    assert not o[0].any() and not o[1, 0].any()
    ctx.close()


def test_topk_at_maximum_context_and_k(ess_lib):
    """one row of 524288 scores (the largest context the library accepts), k = 4096"""
    print("edges: top-k at max_ctx 524288, k 4096", flush=True)
    L, k = 524288, 4096
    rng = np.random.default_rng(5)
    sc = (np.rint(rng.normal(30000, 6000, (1, 1, L))).clip(0) / 16).astype(np.float32)
    ctx = _ctx(max_batch=1, max_q_tokens=1, max_ctx=L, idx_heads=4, idx_dim=32, topk=k, attn_heads=8)
    idx = torch.empty((1, 1, k), dtype=torch.int32, device="cuda")
    for n in (L, L - 3, 70001):
        ctx.topk(torch.from_numpy(sc).cuda(), torch.tensor([n], dtype=torch.int32).cuda(), idx)
        torch.cuda.synchronize()
        ref = O.topk(sc, np.array([n]), k)
        assert np.array_equal(idx.cpu().numpy()[0, 0], np.sort(ref[0, 0])), n
    ctx.close()


def test_bookkeeping_large_pool_path(ess_lib):
    """more than 16384 slots per sequence: stamps are re-read from memory instead of held in registers"""
    from paper_2512_10576_amd import binding as bnd
    print("edges: bookkeeping with 20000 slots", flush=True)
    B, T, L, S, k = 2, 1, 50000, 20000, 2048
    host = synth.latent_rows_fp8(13, B * L).reshape(B, L, 656)
    hp = torch.empty((B, L, 656), dtype=torch.uint8, pin_memory=True)
    hp.copy_(host)
    ctx_len = torch.full((B,), L, dtype=torch.int32)
    ctx = _ctx(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=4, idx_dim=32, topk=k, attn_heads=8, slots_per_seq=S,
               latent_fmt=1)
    cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
    ctx.cache_reset(cache, B)
    oc = O.SlotCache(B, L, S)
    opool = np.zeros((B, S, 656), np.uint8)
    trace = synth.TopkTrace(6, ctx_len, T, k, 0.1, zipf_s=0.2)     # nearly uniform, 90 % new entries per step
    slot_idx = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    mc = torch.empty((B,), dtype=torch.int32, device="cuda")
    for step in range(1, 25):                                   # enough steps to fill the pool and start evicting
        idx = trace.next()
        r = oc.step(idx.numpy(), step)
        O.fill_slots(opool, host.numpy(), r["miss_tok"], r["victims"])
        ctx.gather_latent(cache, idx.cuda(), ctx_len.cuda(), step, slot_idx, None, mc)
        torch.cuda.synchronize()
        assert np.array_equal(mc.cpu().numpy(), r["miss_count"]), step
        assert np.array_equal(slot_idx.cpu().numpy(), r["slot_idx"]), step
        assert np.array_equal(cache.token_of.cpu().numpy(), oc.token_of), step
    assert np.array_equal(cache.slot_pool.cpu().numpy(), opool)
    assert (oc.token_of >= 0).all()                              # the pool filled up, so victims were evicted
    ctx.close()


def test_single_sequence_single_head_block(ess_lib):
    """B = 1, H = 1, k = 1: the smallest shapes"""
    from paper_2512_10576_amd import binding as bnd
    print("edges: B=1 H=1 k=1", flush=True)
    B, T, Hi, Di, L, k, H = 1, 1, 1, 32, 64, 1, 1
    qi, w, key = synth.indexer_inputs(71, B, T, Hi, Di, L, 4, 4, 8)
    ctx_len = torch.tensor([64], dtype=torch.int32)
    pool = synth.latent_rows_bf16(71, L).reshape(1, L, 1152)
    q = synth.attn_query(71, B, T, H)
    oc = O.SlotCache(B, L, L)
    oc.make_resident_identity()
    r = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx_len.numpy(), k, oc, pool.numpy().copy(), None,
                      _qbits(q), O.FMT_BF16, 0.3, 1)
    ctx = _ctx(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H, sm_scale=0.3)
    cache = bnd.Cache.allocate(ctx.cfg, B, slot_pool=pool.cuda())
    ctx.cache_reset(cache, B)
    idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
    out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
    ctx.decode_step(cache, qi.cuda(), w.cuda(), key.cuda(), ctx_len.cuda(), q.cuda(), 1, idx_out, out)
    torch.cuda.synchronize()
    assert idx_out.cpu().numpy().tolist() == r["idx"].tolist()
    # one selected row with softmax weight 1: the output is that row (exactly, it is already bf16)
    row = pool.view(torch.bfloat16).reshape(L, 576)[int(r["idx"][0, 0, 0]), :512].float().numpy()
    assert np.array_equal(out.float().cpu().numpy()[0, 0, 0], row)
    ctx.close()


@pytest.mark.parametrize("B,ctx_lens", [(1, [5000]), (2, [5000, 37]), (5, [5000, 4000, 0, 3000, 2111]), (17, None)])
def test_switch_with_confined_fetches_at_odd_batch_sizes(ess_lib, B, ctx_lens):
    """The overlap switch with a threshold of zero (split batch whenever there are two sequences, fetches
    confined, kernels beside them by ticket) at batch sizes that do not divide evenly, with an empty
    sequence among them, against the plain DA schedule: bit-identical outputs and cache state."""
    from paper_2512_10576_amd import binding as bnd
    print("edges: switch / confinement at batch", B, flush=True)
    T, Hi, Di, L, k, H, S = 2, 64, 128, 5000, 512, 128, 1300
    qi, w, key = synth.indexer_inputs(83, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor(ctx_lens if ctx_lens else [L - 37 * b for b in range(B)], dtype=torch.int32)
    host = synth.latent_rows_bf16(83, B * L).reshape(B, L, 1152)
    hp = torch.empty((B, L, 1152), dtype=torch.uint8, pin_memory=True)
    hp.copy_(host)
    dev = [x.cuda() for x in (qi, w, key, ctx_len)]
    # other index queries for the later steps (same keys): new selections, hence misses in every step
    qws = [(qi.cuda(), w.cuda())] + [tuple(x.cuda() for x in synth.indexer_inputs(83 + s, B, T, Hi, Di, L, 8, 8, 16)[:2])
                                     for s in (1, 2)]
    results, confined, parts = {}, [], []
    for flags in (0, 4):
        ctx = _ctx(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
                   slots_per_seq=S, flags=flags)
        if flags == 4:
            ctx.set_overlap_threshold(0)
        cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp,
                                   slot_pool=torch.full((B, S, 1152), 0x7F, dtype=torch.uint8, device="cuda"))
        ctx.cache_reset(cache, B)
        idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
        out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
        mc = torch.empty((B,), dtype=torch.int32, device="cuda")
        steps = []
        for step in range(1, 4):
            q = synth.attn_query(90 + step, B, T, H)
            ctx.decode_step(cache, qws[step - 1][0], qws[step - 1][1], dev[2], dev[3], q.cuda(), step, idx_out, out, lse, mc)
            torch.cuda.synchronize()
            if flags != 0:
                confined.append(ctx.last_confined())
                parts.append(ctx.last_overlap())
            steps.append((idx_out.clone(), out.clone(), lse.clone(), mc.clone(), cache.slot_of.clone(),
                          cache.slot_pool.clone()))
        assert ctx.get_stats()["steps"] == 3                     # also: no self-check failure pending
        ctx.close()
        results[flags] = steps
    for s0, s4 in zip(results[0], results[4]):
        for x, y in zip(s0, s4):
            assert torch.equal(x, y)
    # step 1 has no miss counts yet (DA, nothing confined); later steps follow steps full of misses, so the
    # fetch is long against everything beside it
    assert confined[0] == 0 and min(confined[1:]) >= 1, confined
    assert parts[1:] == [1 if B >= 2 else 0] * 2, parts


@pytest.mark.parametrize("grid", [1, 2, 7, 8, 24, 0])
def test_ticket_fed_launches_complete_at_any_launch_size(ess_lib, grid):
    """Confined schedules hand their work out by ticket and every working workgroup draws tickets until none is
    left, so the result may not depend on how many workgroups a launch has nor on where the hardware puts
    them.  The test hook fixes the size of every ticket-fed launch (1 = a single workgroup, which then does
    all the work wherever it lands; 0 = the library's own sizing); outputs and cache state equal the plain DA
    schedule bit for bit, and no assertion of the library fires."""
    from paper_2512_10576_amd import binding as bnd
    print("edges: ticket-fed launches with", grid, "workgroups", flush=True)
    B, T, Hi, Di, L, k, H, S = 5, 2, 64, 128, 5000, 512, 128, 1300
    qi, w, key = synth.indexer_inputs(87, B, T, Hi, Di, L, 8, 8, 16)
    ctx_len = torch.tensor([5000, 4000, 0, 3000, 2111], dtype=torch.int32)
    host = synth.latent_rows_bf16(87, B * L).reshape(B, L, 1152)
    hp = torch.empty((B, L, 1152), dtype=torch.uint8, pin_memory=True)
    hp.copy_(host)
    dev = [x.cuda() for x in (qi, w, key, ctx_len)]
    qws = [(qi.cuda(), w.cuda())] + [tuple(x.cuda() for x in synth.indexer_inputs(87 + s, B, T, Hi, Di, L, 8, 8, 16)[:2])
                                     for s in (1, 2)]
    results, confined = {}, []
    for flags in (0, 4, 20):                                     # 20: stages 1-2 in the fused form, four ticket-fed launches
        ctx = _ctx(max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=k, attn_heads=H,
                   slots_per_seq=S, flags=flags)
        if flags != 0:
            ctx.set_overlap_threshold(0)
            ctx.debug_ticket_grid(grid)
        cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp,
                                   slot_pool=torch.full((B, S, 1152), 0x7F, dtype=torch.uint8, device="cuda"))
        ctx.cache_reset(cache, B)
        idx_out = torch.empty((B, T, k), dtype=torch.int32, device="cuda")
        out = torch.empty((B, T, H, 512), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
        mc = torch.empty((B,), dtype=torch.int32, device="cuda")
        steps = []
        for step in range(1, 4):
            q = synth.attn_query(95 + step, B, T, H)
            ctx.decode_step(cache, qws[step - 1][0], qws[step - 1][1], dev[2], dev[3], q.cuda(), step, idx_out, out, lse, mc)
            torch.cuda.synchronize()
            if flags != 0:
                confined.append(ctx.last_confined())
            steps.append((idx_out.clone(), out.clone(), lse.clone(), mc.clone(), cache.slot_of.clone(),
                          cache.token_of.clone(), cache.stamp.clone(), cache.slot_pool.clone()))
        assert ctx.get_stats()["steps"] == 3                     # also: no assertion of a confined step pending
        ctx.close()
        results[flags] = steps
    for other in (4, 20):
        for s0, s4 in zip(results[0], results[other]):
            for x, y in zip(s0, s4):
                assert torch.equal(x, y)
    assert confined[0] == 0 and confined[3] == 0 and min(confined[1:3] + confined[4:]) >= 1, confined


@pytest.mark.parametrize("stride,fmt", [(1152, 0), (656, 1)])
def test_calib_memcpy_rows_delivers_host_pool_rows(ess_lib, stride, fmt):
    """The per-entry copy the paper starts from (Sec. 3.1: one memcpy per block): the rows it delivers are the
    host pool's bytes, and the same entries fetched by the library's own path (ess_gather_latent on an empty
    pool: bookkeeping + fetch kernel reading the pinned pool by address) are the same bytes, which are also
    what the oracle's fill delivers."""
    from paper_2512_10576_amd import binding as bnd
    print("calib_memcpy_rows, entry size", stride, flush=True)
    B, L, k, S = 3, 4096, 300, 640
    rng = np.random.default_rng(21)
    host = torch.from_numpy(rng.integers(0, 256, (B, L, stride), dtype=np.uint8))
    hp = torch.empty((B, L, stride), dtype=torch.uint8, pin_memory=True)
    hp.copy_(host)
    pos = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(B)]).astype(np.int32)     # [B,k]
    flat = torch.from_numpy((pos.astype(np.int64) + np.arange(B)[:, None] * L).reshape(-1)).contiguous()
    dst = torch.full((B * k, stride), 0xEE, dtype=torch.uint8, device="cuda")
    bnd.calib_memcpy_rows(dst, hp, flat, stride, stride)
    torch.cuda.synchronize()
    want = host.numpy().reshape(B * L, stride)[flat.numpy()]
    assert np.array_equal(dst.cpu().numpy(), want)
    # a copy of fewer bytes than the stride leaves the rest of each destination row alone
    dst2 = torch.full((B * k, stride), 0xEE, dtype=torch.uint8, device="cuda")
    bnd.calib_memcpy_rows(dst2, hp, flat, stride - 16, stride)
    torch.cuda.synchronize()
    d2 = dst2.cpu().numpy()
    assert np.array_equal(d2[:, :stride - 16], want[:, :stride - 16]) and np.all(d2[:, stride - 16:] == 0xEE)
    # the library's fetch path on the same entries
    ctx = _ctx(max_batch=B, max_q_tokens=1, max_ctx=L, idx_heads=4, idx_dim=32, topk=k, attn_heads=8, slots_per_seq=S,
               latent_fmt=fmt, row_stride=stride)
    cache = bnd.Cache.allocate(ctx.cfg, B, host_pool=hp)
    ctx.cache_reset(cache, B)
    slot_idx = torch.empty((B, 1, k), dtype=torch.int32, device="cuda")
    rows = torch.empty((B, 1, k, stride), dtype=torch.uint8, device="cuda")
    mc = torch.empty((B,), dtype=torch.int32, device="cuda")
    ctx.gather_latent(cache, torch.from_numpy(pos).reshape(B, 1, k).cuda(), torch.full((B,), L, dtype=torch.int32).cuda(), 1,
                      slot_idx, rows, mc)
    torch.cuda.synchronize()
    assert np.array_equal(rows.cpu().numpy().reshape(B * k, stride), want)
    oc = O.SlotCache(B, L, S)
    opool = np.zeros((B, S, stride), np.uint8)
    r = oc.step(pos.reshape(B, 1, k), 1)
    O.fill_slots(opool, host.numpy(), r["miss_tok"], r["victims"])
    assert np.array_equal(O.gather_rows(opool, r["slot_idx"]).reshape(B * k, stride), want)
    assert np.array_equal(mc.cpu().numpy(), r["miss_count"]) and np.array_equal(cache.slot_pool.cpu().numpy(), opool)
    ctx.close()
    with pytest.raises(bnd.EssError) as ei:                          # a negative row index is refused before any copy
        bnd.calib_memcpy_rows(dst, hp, torch.tensor([3, -1], dtype=torch.int64), stride, stride)
    assert ei.value.code == bnd.ESS_ERR_INVALID_ARG


def test_calib_read_reads_every_byte_once(ess_lib):
    """The plain read kernel that measures the achievable read rate: its checksum (xor of all 32-bit words, one
    partial word per workgroup) equals the xor computed on the host, for sizes with ragged ends."""
    from paper_2512_10576_amd import binding as bnd
    rng = np.random.default_rng(3)
    for n_bytes in (16, 4096 + 16, 3 * 262144 + 48, 40 * 1000 * 1000):
        print("calib_read", n_bytes, flush=True)
        host = rng.integers(0, 256, n_bytes, dtype=np.uint8)
        sink = torch.zeros(bnd.CALIB_READ_WGS, dtype=torch.int32, device="cuda")
        bnd.calib_read(torch.from_numpy(host).cuda(), sink)
        torch.cuda.synchronize()
        got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        assert got == np.bitwise_xor.reduce(host.view(np.uint32))
