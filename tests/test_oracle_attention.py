"""Pins for the oracle's sparse MLA decode and merge (CPU only): dense masked
attention through torch's scaled_dot_product_attention, closed forms, invariants."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth


def _setup(seed, B, T, H, L, k):
    q = synth.attn_query(seed, B, T, H)
    pool = synth.latent_rows_bf16(seed, B * L).reshape(B, L, 1152)
    rng = np.random.default_rng(seed)
    idx = np.stack([np.stack([rng.choice(L, k, replace=False) for _ in range(T)]) for _ in range(B)]).astype(np.int32)
    return q, pool, idx


def _qbits(q):
    return q.view(torch.int16).numpy().view(np.uint16)


def test_sparse_equals_dense_attention_with_topk_mask():
    B, T, H, L, k = 2, 2, 5, 96, 20
    q, pool, idx = _setup(1, B, T, H, L, k)
    idx[1, 0, -4:] = -1
    scale = 0.37
    out, lse = O.sparse_mla(_qbits(q), pool.numpy(), idx, O.FMT_BF16, scale)
    rows = pool.view(torch.bfloat16).reshape(B, L, 576).to(torch.float64)
    for b in range(B):
        for t in range(T):
            mask = torch.full((L,), float("-inf"), dtype=torch.float64)
            sel = idx[b, t][idx[b, t] >= 0]
            mask[torch.as_tensor(sel, dtype=torch.long)] = 0.0
            ref = F.scaled_dot_product_attention(
                q[b, t].to(torch.float64).unsqueeze(0), rows[b].unsqueeze(0), rows[b, :, :512].unsqueeze(0),
                attn_mask=mask.expand(H, L).unsqueeze(0), scale=scale)[0]
            assert np.allclose(out[b, t], ref.numpy(), rtol=1e-12, atol=1e-12)
            z = scale * (q[b, t].to(torch.float64) @ rows[b].T) + mask
            assert np.allclose(lse[b, t], torch.logsumexp(z, dim=1).numpy(), rtol=1e-12, atol=1e-12)


def test_all_rows_selected_is_ordinary_attention():
    B, T, H, L = 1, 1, 3, 33
    q, pool, _ = _setup(2, B, T, H, L, 1)
    idx = np.arange(L, dtype=np.int32).reshape(1, 1, L)
    out, _ = O.sparse_mla(_qbits(q), pool.numpy(), idx, O.FMT_BF16, 1 / 24.0)
    rows = pool.view(torch.bfloat16).reshape(B, L, 576).to(torch.float64)
    ref = F.scaled_dot_product_attention(q[0].to(torch.float64), rows, rows[..., :512], scale=1 / 24.0)
    assert np.allclose(out[0, 0], ref[0].numpy(), rtol=1e-12, atol=1e-12)


def test_closed_forms():
    B, T, H, L, k = 1, 1, 4, 40, 9
    q, pool, idx = _setup(3, B, T, H, L, k)
    rows = O.decode_rows(pool.numpy(), O.FMT_BF16)
    # zero query: uniform softmax => mean of the selected rows, lse = log k
    q0 = np.zeros((B, T, H, 576), np.uint16)
    out, lse = O.sparse_mla(q0, pool.numpy(), idx, O.FMT_BF16, 1.0)
    assert np.allclose(out[0, 0, 0], rows[0, idx[0, 0], :512].mean(axis=0), atol=1e-14)
    assert np.allclose(lse, np.log(k))
    # identical rows: output is that row whatever the query
    same = pool.clone()
    same[0, :] = pool[0, 5]
    out, _ = O.sparse_mla(_qbits(q), same.numpy(), idx, O.FMT_BF16, 0.2)
    assert np.allclose(out[0, 0], np.broadcast_to(rows[0, 5, :512], (H, 512)), atol=1e-13)
    # softmax weights sum to one: rows whose value part is all ones give all ones
    ones = pool.clone().view(torch.bfloat16).reshape(B, L, 576)
    ones[..., :512] = 1.0
    out, _ = O.sparse_mla(_qbits(q), ones.view(torch.uint8).reshape(B, L, 1152).numpy(), idx, O.FMT_BF16, 0.2)
    assert np.allclose(out, 1.0, atol=1e-14)
    # empty selection
    out, lse = O.sparse_mla(_qbits(q), pool.numpy(), np.full((1, 1, 4), -1, np.int32), O.FMT_BF16, 0.2)
    assert not out.any() and np.all(np.isneginf(lse))
    # very peaky softmax picks the best-matching row
    out, _ = O.sparse_mla(_qbits(q), pool.numpy(), idx, O.FMT_BF16, 50.0)
    z = O.decode_bf16(_qbits(q))[0, 0] @ rows[0, idx[0, 0]].T
    assert np.allclose(out[0, 0], rows[0, idx[0, 0][z.argmax(axis=1)], :512], atol=1e-6)


def test_permutation_and_split_merge():
    B, T, H, L, k = 2, 1, 6, 64, 24
    q, pool, idx = _setup(4, B, T, H, L, k)
    full, lfull = O.sparse_mla(_qbits(q), pool.numpy(), idx, O.FMT_BF16, 0.1)
    perm = idx[:, :, ::-1].copy()
    o2, l2 = O.sparse_mla(_qbits(q), pool.numpy(), perm, O.FMT_BF16, 0.1)
    assert np.allclose(full, o2, atol=1e-13) and np.allclose(lfull, l2, atol=1e-13)
    for cut in (0, 1, 7, k):
        a, b_ = idx.copy(), idx.copy()
        a[:, :, cut:] = -1
        b_[:, :, :cut] = -1
        o0, l0 = O.sparse_mla(_qbits(q), pool.numpy(), a, O.FMT_BF16, 0.1)
        o1, l1 = O.sparse_mla(_qbits(q), pool.numpy(), b_, O.FMT_BF16, 0.1)
        om, lm = O.merge_partials(o0, l0, o1, l1)
        assert np.allclose(om, full, atol=1e-13) and np.allclose(lm, lfull, atol=1e-13)
    e_o, e_l = O.merge_partials(np.zeros((1, 2)), [-np.inf], np.zeros((1, 2)), [-np.inf])
    assert not e_o.any() and np.isneginf(e_l[0])


def test_fp8_rows_attention_matches_dense_library_attention():
    B, T, H, L = 1, 1, 4, 48
    q = synth.attn_query(8, B, T, H)
    pool = synth.latent_rows_fp8(8, L).reshape(1, L, 656)
    idx = np.arange(L, dtype=np.int32).reshape(1, 1, L)
    out, _ = O.sparse_mla(_qbits(q), pool.numpy(), idx, O.FMT_FP8, 1 / 24.0)
    lat = pool[0, :, :512].contiguous().view(torch.float8_e4m3fn).to(torch.float64).reshape(L, 4, 128)
    sc = pool[0, :, 512:520].contiguous().view(torch.bfloat16).to(torch.float64)
    rope = pool[0, :, 520:648].contiguous().view(torch.bfloat16).to(torch.float64)
    v = (lat * sc.unsqueeze(-1)).reshape(L, 512)
    kk = torch.cat([v, rope], dim=1)
    ref = F.scaled_dot_product_attention(q[0].to(torch.float64), kk.unsqueeze(0), v.unsqueeze(0), scale=1 / 24.0)
    assert np.allclose(out[0, 0], ref[0].numpy(), rtol=1e-12, atol=1e-12)


def test_decode_step_is_the_stages_in_sequence_and_offload_is_lossless():
    B, T, Hi, Di, L, k, H = 2, 2, 4, 32, 512, 32, 4
    qi, w, key = synth.indexer_inputs(21, B, T, Hi, Di, L, 4, 4, 8)
    ctx = np.array([512, 400], np.int32)
    q = synth.attn_query(21, B, T, H)
    host = synth.latent_rows_bf16(21, B * L).reshape(B, L, 1152).numpy()
    # offloaded: 25 % slots
    S = 128
    c = O.SlotCache(B, L, S)
    pool = np.zeros((B, S, 1152), np.uint8)
    # resident
    cr = O.SlotCache(B, L, L)
    cr.make_resident_identity()
    poolr = host.copy()
    for step in (1, 2, 3):
        r = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx, k, c, pool, host, _qbits(q), O.FMT_BF16, 1 / 24.0, step)
        rr = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx, k, cr, poolr, None, _qbits(q), O.FMT_BF16, 1 / 24.0, step)
        assert np.array_equal(r["idx"], rr["idx"])
        assert np.array_equal(r["out"], rr["out"]) and np.array_equal(r["lse"], rr["lse"])
        sc = O.index_score(qi.numpy(), w.numpy(), key.numpy(), ctx)
        ix = O.topk(sc, ctx, k)
        assert np.array_equal(r["idx"], ix)
        o, l = O.sparse_mla(_qbits(q), host, ix, O.FMT_BF16, 1 / 24.0)   # attention straight from the host pool
        assert np.array_equal(o, r["out"]) and np.array_equal(l, r["lse"])
        assert (r["miss_count"].sum() > 0) == (step == 1)
        # T=2 causal offset: query 0 never selects the newest position
        assert (ix[:, 0] != (ctx - 1)[:, None]).all()
    # override drives stages 3-5 while stages 1-2 still report their own result
    ov = np.stack([np.stack([np.arange(t, t + k) for t in range(T)]) for _ in range(B)]).astype(np.int32)
    r = O.decode_step(qi.numpy(), w.numpy(), key.numpy(), ctx, k, c, pool, host, _qbits(q), O.FMT_BF16, 1 / 24.0, 4, topk_override=ov)
    assert np.array_equal(r["idx"], ix) and np.array_equal(r["used_idx"], ov)
    o, _ = O.sparse_mla(_qbits(q), host, ov, O.FMT_BF16, 1 / 24.0)
    assert np.array_equal(o, r["out"])
