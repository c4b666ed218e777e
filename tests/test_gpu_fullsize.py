"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the GPU result
of sampled sequences is checked against the CPU oracle one by one, plus properties that hold for the
whole batch.  Inputs come from bench.build_workload (seeded, synthetic)."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O

pytestmark = pytest.mark.gpu


def _qbits(q):
    return q.view(torch.int16).cpu().numpy().view(np.uint16)


def _attn_close(got_bf16, ref):
    got = got_bf16.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= 2e-2 + 2e-2 * np.abs(ref))
    assert err.max() <= 3e-3, err.max()
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-2


def test_cfg2_full_size_sampled_sequences(ess_lib):
    import bench
    print("full-size cfg2 (B32, ctx 32768, resident)", flush=True)
    W = bench.build_workload("cfg2", 0)
    wl, ctx = W["wl"], W["ctx"]
    B, L, k, H = wl["B"], wl["L"], wl["k"], wl["H"]
    score = torch.empty((B, 1, L), dtype=torch.float32, device="cuda")
    ctx.index_score(W["q_idx"], W["w"], W["key"], W["ctx_len"], score)
    bench.run_steps(W, 1, 1)
    torch.cuda.synchronize()
    idx_gpu = W["idx_out"].cpu().numpy()
    assert int(W["miss"].sum().item()) == 0
    for b in (0, 17, 31):
        print("  sequence", b, flush=True)
        q_idx = W["q_idx"][b:b + 1].cpu().numpy(); w = W["w"][b:b + 1].cpu().numpy()
        key = W["key"][b:b + 1].cpu().numpy(); cl = W["ctx_len"][b:b + 1].cpu().numpy()
        ref_score = O.index_score(q_idx, w, key, cl)
        assert np.array_equal(score[b].cpu().numpy(), ref_score[0])                    # bit-exact scores
        ref_idx = O.topk(ref_score, cl, k)
        assert np.array_equal(idx_gpu[b, 0], np.sort(ref_idx[0, 0]))                   # bit-exact selection
        pool = W["cache"].slot_pool[b:b + 1].cpu().numpy()
        ref_out, _ = O.sparse_mla(_qbits(W["q_attn"][b:b + 1]), pool, ref_idx, O.FMT_BF16, 576 ** -0.5)
        _attn_close(W["out"][b:b + 1], ref_out)
    # whole batch: every row holds k distinct ascending visible positions
    assert np.all(np.diff(idx_gpu[:, 0, :], axis=1) > 0) and idx_gpu.min() >= 0 and idx_gpu.max() < L
    ctx.close()


def test_cfg4_full_size_sampled_sequences(ess_lib):
    import bench
    print("full-size cfg4 (B64, ctx up to 131072, offloaded, trace-driven)", flush=True)
    steps = 3
    W = bench.build_workload("cfg4", steps)
    wl, ctx, cache = W["wl"], W["ctx"], W["cache"]
    B, L, k, S = wl["B"], wl["L"], wl["k"], W["S"]
    sample = (0, 40, 63)
    oracles = {b: (O.SlotCache(1, L, S), np.zeros((1, S, 1152), np.uint8)) for b in sample}
    lens = W["ctx_len"].cpu().numpy()
    schedules = []
    for step in range(1, steps + 1):
        bench.run_steps(W, step, 1)
        torch.cuda.synchronize()
        ov = W["trace"][step - 1].cpu().numpy()
        slot_of = cache.slot_of.cpu().numpy(); token_of = cache.token_of.cpu().numpy()
        stamp = cache.stamp.cpu().numpy().view(np.uint32); miss = W["miss"].cpu().numpy()
        for b in sample:
            print("  step", step, "sequence", b, flush=True)
            oc, opool = oracles[b]
            host = W["host_pool"][b:b + 1].numpy()
            r = oc.step(ov[b:b + 1], step)
            O.fill_slots(opool, host, r["miss_tok"], r["victims"])
            assert miss[b] == r["miss_count"][0]
            assert np.array_equal(slot_of[b], oc.slot_of[0]) and np.array_equal(token_of[b], oc.token_of[0])
            assert np.array_equal(stamp[b], oc.stamp[0])
            occ = np.nonzero(oc.token_of[0] >= 0)[0]
            gpu_rows = cache.slot_pool[b].cpu().numpy()
            assert np.array_equal(gpu_rows[occ], opool[0, occ])                         # fetched bytes == host bytes
            ref_out, _ = O.sparse_mla(_qbits(W["q_attn"][b:b + 1]), opool, r["slot_idx"], O.FMT_BF16, 576 ** -0.5)
            _attn_close(W["out"][b:b + 1], ref_out)
            if step == 1:                                                                # stages 1-2 ran on the real data
                q_idx = W["q_idx"][b:b + 1].cpu().numpy(); w = W["w"][b:b + 1].cpu().numpy()
                key = W["key"][b:b + 1].cpu().numpy()
                ref_idx = O.topk(O.index_score(q_idx, w, key, lens[b:b + 1]), lens[b:b + 1], k)
                assert np.array_equal(W["idx_out"][b, 0].cpu().numpy(), np.sort(ref_idx[0, 0]))
        # whole batch: the selection is resident after the step; tables are mutually inverse
        sel = torch.from_numpy(ov[:, 0, :].astype(np.int64)).cuda()
        assert bool((torch.gather(cache.slot_of, 1, sel) >= 0).all())
        res = cache.token_of >= 0
        back = torch.gather(cache.slot_of, 1, cache.token_of.clamp(min=0).long())
        assert bool((back[res] == torch.arange(S, device="cuda").expand(B, S)[res]).all())
        schedules.append((ctx.last_overlap(), ctx.last_confined()))
    ctx.close()
    # the launch configuration bench.py times: split batch, both fetches confined, kernels beside them by ticket
    assert schedules[0] == (0, 0) and schedules[-1] == (1, 2), schedules


def test_cfg3_full_size_sampled_sequences(ess_lib):
    """B64, context 32768, 25 % slots, 80 % step-to-step overlap, in the schedule bench.py runs there: the switch
    stays with DA (half a batch's index score at 32K is too short to be worth splitting) and confines the fetch."""
    import bench
    print("full-size cfg3 (B64, ctx 32768, offloaded, 25% slots, trace-driven)", flush=True)
    steps = 3
    W = bench.build_workload("cfg3", steps)
    wl, ctx, cache = W["wl"], W["ctx"], W["cache"]
    B, L, k, S = wl["B"], wl["L"], wl["k"], W["S"]
    assert (B, L, S, W["stride"]) == (64, 32768, 8192, 1152)
    sample = (0, 29, 63)
    oracles = {b: (O.SlotCache(1, L, S), np.zeros((1, S, 1152), np.uint8)) for b in sample}
    lens = W["ctx_len"].cpu().numpy()
    schedules = []
    for step in range(1, steps + 1):
        bench.run_steps(W, step, 1)
        torch.cuda.synchronize()
        ov = W["trace"][step - 1].cpu().numpy()
        slot_of = cache.slot_of.cpu().numpy(); token_of = cache.token_of.cpu().numpy()
        stamp = cache.stamp.cpu().numpy().view(np.uint32); miss = W["miss"].cpu().numpy()
        for b in sample:
            print("  step", step, "sequence", b, flush=True)
            oc, opool = oracles[b]
            host = W["host_pool"][b:b + 1].numpy()
            r = oc.step(ov[b:b + 1], step)
            O.fill_slots(opool, host, r["miss_tok"], r["victims"])
            assert miss[b] == r["miss_count"][0]
            assert np.array_equal(slot_of[b], oc.slot_of[0]) and np.array_equal(token_of[b], oc.token_of[0])
            assert np.array_equal(stamp[b], oc.stamp[0])
            occ = np.nonzero(oc.token_of[0] >= 0)[0]
            gpu_rows = cache.slot_pool[b].cpu().numpy()
            assert np.array_equal(gpu_rows[occ], opool[0, occ])
            ref_out, _ = O.sparse_mla(_qbits(W["q_attn"][b:b + 1]), opool, r["slot_idx"], O.FMT_BF16, 576 ** -0.5)
            _attn_close(W["out"][b:b + 1], ref_out)
            if step == 1:
                q_idx = W["q_idx"][b:b + 1].cpu().numpy(); w = W["w"][b:b + 1].cpu().numpy()
                key = W["key"][b:b + 1].cpu().numpy()
                ref_idx = O.topk(O.index_score(q_idx, w, key, lens[b:b + 1]), lens[b:b + 1], k)
                assert np.array_equal(W["idx_out"][b, 0].cpu().numpy(), np.sort(ref_idx[0, 0]))
        sel = torch.from_numpy(ov[:, 0, :].astype(np.int64)).cuda()
        assert bool((torch.gather(cache.slot_of, 1, sel) >= 0).all())
        res = cache.token_of >= 0
        back = torch.gather(cache.slot_of, 1, cache.token_of.clamp(min=0).long())
        assert bool((back[res] == torch.arange(S, device="cuda").expand(B, S)[res]).all())
        schedules.append((ctx.last_overlap(), ctx.last_confined()))
    assert ctx.get_stats()["steps"] == steps
    ctx.close()
    # the launch configuration bench.py times here: DA, the fetch confined, Attn0 beside it by ticket
    assert schedules[0] == (0, 0) and schedules[-1] == (0, 1), schedules


def test_cfg5_full_size_sampled_sequences(ess_lib):
    """Multi-token decode at full size: batch 128, two query tokens with the causal offset, quantised
    entries (656 bytes), one of the 61 layers (the layers differ only in their seeds)."""
    import bench
    print("full-size cfg5 (B128, T2, ctx 131072, fp8 entries, offloaded, trace-driven)", flush=True)
    steps = 2
    W = bench.build_workload("cfg5", steps, layers=1)
    wl, ctx, cache = W["wl"], W["ctx"], W["cache"]
    B, T, L, k, S = wl["B"], wl["T"], wl["L"], wl["k"], W["S"]
    assert (B, T, W["stride"], W["fmt"]) == (128, 2, 656, 1)
    sample = (0, 77, 127)
    oracles = {b: (O.SlotCache(1, L, S), np.zeros((1, S, 656), np.uint8)) for b in sample}
    lens = W["ctx_len"].cpu().numpy()
    for step in range(1, steps + 1):
        bench.run_steps(W, step, 1)
        torch.cuda.synchronize()
        ov = W["trace"][step - 1].cpu().numpy()
        slot_of = cache.slot_of.cpu().numpy(); token_of = cache.token_of.cpu().numpy()
        stamp = cache.stamp.cpu().numpy().view(np.uint32); miss = W["miss"].cpu().numpy()
        for b in sample:
            print("  step", step, "sequence", b, flush=True)
            oc, opool = oracles[b]
            host = W["host_pool"][b:b + 1].numpy()
            r = oc.step(ov[b:b + 1], step)
            O.fill_slots(opool, host, r["miss_tok"], r["victims"])
            assert miss[b] == r["miss_count"][0]
            assert np.array_equal(slot_of[b], oc.slot_of[0]) and np.array_equal(token_of[b], oc.token_of[0])
            assert np.array_equal(stamp[b], oc.stamp[0])
            occ = np.nonzero(oc.token_of[0] >= 0)[0]
            gpu_rows = cache.slot_pool[b].cpu().numpy()
            assert np.array_equal(gpu_rows[occ], opool[0, occ])
            ref_out, _ = O.sparse_mla(_qbits(W["q_attn"][b:b + 1]), opool, r["slot_idx"], O.FMT_FP8, 576 ** -0.5)
            _attn_close(W["out"][b:b + 1], ref_out)
            if step == 1:                                                                # both query tokens, causal offset
                q_idx = W["q_idx"][b:b + 1].cpu().numpy(); w = W["w"][b:b + 1].cpu().numpy()
                key = W["key"][b:b + 1].cpu().numpy()
                ref_idx = O.topk(O.index_score(q_idx, w, key, lens[b:b + 1]), lens[b:b + 1], k)
                for t in range(T):
                    assert np.array_equal(W["idx_out"][b, t].cpu().numpy(), np.sort(ref_idx[0, t]))
        sel = torch.from_numpy(ov.reshape(B, T * k).astype(np.int64)).cuda()
        assert bool((torch.gather(cache.slot_of, 1, sel) >= 0).all())
    schedule = (ctx.last_overlap(), ctx.last_confined())
    ctx.close()
    assert schedule[0] == 1 and schedule[1] >= 1, schedule     # split batch with a confined fetch, as bench.py runs it
