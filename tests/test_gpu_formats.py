"""GPU parity of the index score over the whole E4M3 value range.

The benchmark inputs are small integers, which use a handful of E4M3 bit patterns.  Here every finite
pattern (254 of the 256: subnormals, +-0, +-448, every exponent) goes through the fp8 matrix-core path on
both operands:

  * one-hot inputs: every key and every query head holds a single non-zero element, placed so that a
    key meets exactly one head, so each score is w * max(0, q_val * k_val) -- one product of two 4-bit
    significands, exact in float32 whatever the order of summation -- and is compared BIT FOR BIT with
    the oracle, for all 254 x 254 pairs of patterns, at every supported key width, for one and two
    query tokens, over the flat and the paged Indexer-Cache;
  * dense random finite patterns: compared with the float64 oracle within the bound that the matrix core's
    aligned addition gives (the sums are no longer exact), and bit for bit where the magnitudes stay in a
    narrow range."""
import numpy as np
import pytest
import torch

from oracle import ess_oracle as O
from paper_2512_10576_amd import synth
from tests.test_gpu_stages import _ctx

pytestmark = pytest.mark.gpu

FINITE = np.array([b for b in range(256) if b not in (0x7F, 0xFF)], dtype=np.uint8)     # 254 patterns


def _one_hot_inputs(Di, Hi, B, T, seed):
    """keys: token s = d * 254 + p holds pattern FINITE[p] at dimension d (L = Di * 254 tokens, the same for
    every sequence).  queries: head j of row (b,t) holds one pattern at dimension dim(t,j) = j * (Di // Hi) +
    (t % (Di // Hi)), distinct per head; the rows' heads run through all 254 patterns (and wrap).  Weights are
    powers of two."""
    rng = np.random.default_rng(seed)
    L = Di * 254
    key = np.zeros((B, L, Di), np.uint8)
    d_of = np.arange(L) // 254
    key[:, np.arange(L), d_of] = FINITE[np.arange(L) % 254]
    q = np.zeros((B, T, Hi, Di), np.uint8)
    step = Di // Hi
    n = 0
    for b in range(B):
        for t in range(T):
            for j in range(Hi):
                q[b, t, j, j * step + (t % step)] = FINITE[(n * 37 + 11) % 254]       # 37 is coprime to 254: a permutation
                n += 1
    w = (2.0 ** rng.integers(-3, 3, (B, T, Hi))).astype(np.float32)
    return q, w, key, L, n


@pytest.mark.parametrize("Di,Hi,B,T,paged", [
    (32, 32, 8, 1, False), (32, 32, 4, 2, False), (64, 64, 4, 1, False), (64, 32, 4, 2, False),
    (128, 64, 4, 1, False), (128, 64, 2, 2, False), (128, 64, 2, 2, True), (32, 32, 8, 1, True), (64, 64, 2, 2, True),
])
def test_index_score_all_e4m3_patterns_bit_exact(ess_lib, Di, Hi, B, T, paged):
    print("index score, every finite E4M3 pattern: Di", Di, "Hi", Hi, "B", B, "T", T, "paged" if paged else "flat", flush=True)
    q, w, key, L, n_heads = _one_hot_inputs(Di, Hi, B, T, 5 + Di + T)
    assert n_heads >= 254                                                # every pattern appears on the query side
    Lmax = (L + 63) // 64 * 64
    keyp = np.zeros((B, Lmax, Di), np.uint8)
    keyp[:, :L] = key
    lens = np.array([L - 3 * b for b in range(B)], dtype=np.int32)       # ragged tails
    lens[0] = L
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=Lmax, idx_heads=Hi, idx_dim=Di, topk=8, attn_heads=8)
    score = torch.full((B, T, Lmax), -7.0, dtype=torch.float32, device="cuda")
    tq, tw, tl = torch.from_numpy(q).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(lens).cuda()
    if paged:
        pages, table, _ = synth.paged_indexer_cache(90 + Di, torch.from_numpy(keyp), torch.from_numpy(lens), n_spare_pages=3)
        ref = O.index_score_paged(q, w, pages.numpy(), table.numpy(), lens)
        ctx.index_score_paged(tq, tw, pages.cuda(), table.cuda(), tl, score)
    else:
        ref = O.index_score(q, w, keyp, lens)
        ctx.index_score(tq, tw, torch.from_numpy(keyp).cuda(), tl, score)
    torch.cuda.synchronize()
    got = score.cpu().numpy()
    nonzero = 0
    for b in range(B):
        for t in range(T):
            vis = max(int(lens[b]) - (T - 1 - t), 0)
            g, r = got[b, t, :vis], ref[b, t, :vis]
            bad = np.nonzero(g != r)[0]                                  # numeric equality: +0 == -0
            assert bad.size == 0, (b, t, bad[:8], g[bad[:8]], r[bad[:8]])
            nonzero += int(np.count_nonzero(r))
    # the case is not vacuous: about a quarter of the (head, key) pairs give a positive product
    assert nonzero > B * T * Hi * 254 // 5
    # the smallest and the largest products both occur among the references
    pos = ref[np.isfinite(ref) & (ref > 0)]
    assert pos.min() <= 2.0 ** -18 * 4 and pos.max() >= 448.0 * 448.0 / 8
    ctx.close()


@pytest.mark.parametrize("Di,Hi,T", [(128, 64, 1), (128, 64, 2), (64, 40, 1), (32, 4, 2)])
def test_index_score_dense_random_e4m3_within_matrix_core_bound(ess_lib, Di, Hi, T):
    """Every element a random finite pattern, magnitudes from 2^-9 to 448, so the products of one dot product
    span 36 binary orders.  The fp8 matrix core forms the products exactly but adds them after aligning them to
    the largest one, keeping a limited number of bits below it: measured on gfx950 the sum of one instruction
    (32 or 128 terms) is off by up to 2^-11.1 of its largest product, and it is exact when the products lie
    within a few thousand of each other (the benchmark's integer inputs: within 64).  The oracle sums in float64.
    Bound per score: 2^-10 * sum_j w_j * max_d |q_jd * k_sd| (twice the measured worst case per dot product;
    the float32 roundings of the head sum are far below it).  Decoding of every pattern is checked exactly by the
    one-hot test above; this case checks the dense accumulation, ragged tails included."""
    print("index score, dense random E4M3: Di", Di, "Hi", Hi, "T", T, flush=True)
    rng = np.random.default_rng(100 + Di + T)
    B, L = 3, 3000
    q = FINITE[rng.integers(0, 254, (B, T, Hi, Di))]
    key = FINITE[rng.integers(0, 254, (B, L, Di))]
    w = (rng.integers(1, 9, (B, T, Hi)) / 16.0).astype(np.float32)
    lens = np.array([L, 2049, 777], dtype=np.int32)
    ref = O.index_score(q, w, key, lens).astype(np.float64)
    qa, ka = np.abs(O.decode_e4m3(q)), np.abs(O.decode_e4m3(key))
    ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=8, attn_heads=8)
    score = torch.empty((B, T, L), dtype=torch.float32, device="cuda")
    ctx.index_score(torch.from_numpy(q).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(key).cuda(),
                    torch.from_numpy(lens).cuda(), score)
    torch.cuda.synchronize()
    got = score.cpu().numpy().astype(np.float64)
    worst = 0.0
    for b in range(B):
        for t in range(T):
            vis = max(int(lens[b]) - (T - 1 - t), 0)
            # largest product of every (key, head) dot product, weighted: [vis]
            mx = np.stack([(ka[b, :vis] * qa[b, t, j][None, :]).max(axis=1) for j in range(Hi)], axis=1) @ w[b, t].astype(np.float64)
            err = np.abs(got[b, t, :vis] - ref[b, t, :vis])
            worst = max(worst, float((err / mx).max()))
            assert np.all(err <= 2.0 ** -10 * mx), (b, t, worst)
            assert np.count_nonzero(ref[b, t, :vis]) > vis // 2
    print("  largest error / bound: %.3f" % (worst * 2.0 ** 10), flush=True)
    ctx.close()


def test_index_score_dense_e4m3_exact_within_narrow_range(ess_lib):
    """Dense random patterns whose magnitudes lie within a factor 16 of each other (exponent fields 7..10, all
    mantissas, both signs): the products of a dot product lie within 2^9 of each other and their exact sum has at
    most 19 significant bits, so the matrix core's aligned sum is exact.  One head with weight 1: the score is the
    ReLU of one exact dot product, compared bit for bit."""
    print("index score, dense E4M3 in a narrow range: exact", flush=True)
    rng = np.random.default_rng(77)
    pats = np.array([x for x in range(256) if 0x38 <= (x & 0x7F) < 0x58], dtype=np.uint8)
    for Di in (32, 64, 128):
        B, T, Hi, L = 2, 2, 1, 4100
        q = pats[rng.integers(0, len(pats), (B, T, Hi, Di))]
        key = pats[rng.integers(0, len(pats), (B, L, Di))]
        w = np.ones((B, T, Hi), np.float32)
        lens = np.array([L, 1234], dtype=np.int32)
        ref = O.index_score(q, w, key, lens)
        ctx = _ctx(ess_lib, max_batch=B, max_q_tokens=T, max_ctx=L, idx_heads=Hi, idx_dim=Di, topk=8, attn_heads=8)
        score = torch.empty((B, T, L), dtype=torch.float32, device="cuda")
        ctx.index_score(torch.from_numpy(q).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(key).cuda(),
                        torch.from_numpy(lens).cuda(), score)
        torch.cuda.synchronize()
        got = score.cpu().numpy()
        for b in range(B):
            for t in range(T):
                vis = max(int(lens[b]) - (T - 1 - t), 0)
                assert np.array_equal(got[b, t, :vis], ref[b, t, :vis]), (Di, b, t)
        ctx.close()
