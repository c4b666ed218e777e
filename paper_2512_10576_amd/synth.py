"""Seeded synthetic inputs for the ESS decode-step path.

This module only *draws inputs*: random integers, normal values, context
lengths and top-k access traces, and packs them into the byte layouts the
library and the tests agree on.  It holds none of the method's arithmetic
(no score, no selection, no attention, no cache policy); format conversions
go through torch's own casts.  Both the HIP path's callers and the CPU tests
use it, and it imports neither.

The shapes and distributions stand in for DeepSeek-V3.2-Exp activations and
for the LongBench-V2 access pattern the paper analysed (Sec. 2.2), neither
of which is available: indexer q/k are small integers (exact in E4M3),
latent rows are N(0,1), and step-to-step top-k sets have an exact
Intra-Layer Similarity (Eq. 1) with a Zipf-skewed preference for recent
positions.
"""
from __future__ import annotations

import torch

LATENT_DIM = 512
ROPE_DIM = 64
ROW_DIM = 576
ROW_BYTES_BF16 = 1152
ROW_BYTES_FP8 = 648
ROW_STRIDE_FP8 = 656   # the paper's entry size (Sec. 3.1); 8 bytes of zero padding


def _gen(seed: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def indexer_inputs(seed, B, T, Hi, Di, Lmax, qk_max, w_levels, w_den, device="cpu"):
    """q uint8 [B,T,Hi,Di], w float32 [B,T,Hi], key uint8 [B,Lmax,Di].
    q and key are integers uniform in [-qk_max, qk_max] stored as E4M3 bytes;
    w is uniform in {1..w_levels}/w_den."""
    g = _gen(seed, device)
    qi = torch.randint(-qk_max, qk_max + 1, (B, T, Hi, Di), generator=g, device=device)
    wi = torch.randint(1, w_levels + 1, (B, T, Hi), generator=g, device=device)
    q = qi.to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8)
    w = wi.to(torch.float32) / float(w_den)
    key = torch.empty((B, Lmax, Di), dtype=torch.uint8, device=device)
    for b in range(B):  # one sequence at a time bounds the int64 temporary
        ki = torch.randint(-qk_max, qk_max + 1, (Lmax, Di), generator=g, device=device)
        key[b] = ki.to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8)
    return q, w, key


def attn_query(seed, B, T, H, device="cpu"):
    """Absorbed attention queries, N(0,1) rounded to bfloat16: [B,T,H,576] bf16."""
    g = _gen(seed + 7919, device)
    return torch.randn((B, T, H, ROW_DIM), generator=g, device=device).to(torch.bfloat16)


def latent_rows_bf16(seed, n_rows, device="cpu", out=None):
    """n_rows Latent-Cache entries, N(0,1) bf16, as bytes [n_rows,1152]."""
    g = _gen(seed + 104729, device)
    x = torch.randn((n_rows, ROW_DIM), generator=g, device=device).to(torch.bfloat16)
    b = x.view(torch.uint8).reshape(n_rows, ROW_BYTES_BF16)
    if out is not None:
        out.copy_(b)
        return out
    return b


def latent_rows_fp8(seed, n_rows, device="cpu"):
    """n_rows entries in the quantised layout, as bytes [n_rows,656]:
    [0,512) E4M3 latent, [512,520) 4 bf16 scales (amax/448 per 128 elements),
    [520,648) 64 bf16 rope, [648,656) zero."""
    g = _gen(seed + 1299709, device)
    lat = torch.randn((n_rows, 4, 128), generator=g, device=device)
    rope = torch.randn((n_rows, ROPE_DIM), generator=g, device=device).to(torch.bfloat16)
    scale = (lat.abs().amax(dim=-1) / 448.0).to(torch.bfloat16)
    scale = torch.where(scale == 0, torch.ones_like(scale), scale)
    qv = (lat / scale.to(torch.float32).unsqueeze(-1)).clamp(-448.0, 448.0).to(torch.float8_e4m3fn)
    rows = torch.zeros((n_rows, ROW_STRIDE_FP8), dtype=torch.uint8, device=device)
    rows[:, :512] = qv.view(torch.uint8).reshape(n_rows, 512)
    rows[:, 512:520] = scale.view(torch.uint8).reshape(n_rows, 8)
    rows[:, 520:648] = rope.view(torch.uint8).reshape(n_rows, 128)
    return rows


def ctx_lengths(seed, B, lo, hi, device="cpu"):
    """Per-sequence context lengths, uniform integers in [lo, hi]; int32 [B]."""
    g = _gen(seed + 15485863, device)
    return torch.randint(lo, hi + 1, (B,), generator=g, device=device).to(torch.int32)


class TopkTrace:
    """Step-to-step top-k index sets with an exact overlap.

    Step 0 draws k distinct visible positions without replacement with
    probability proportional to (r+1)^(-zipf_s), r = distance from the newest
    visible position (Gumbel-top-k sampling).  Every later step keeps
    floor(rho*k) uniformly chosen members of the previous set and draws the
    rest, with the same weights, from positions outside the previous set, so
    |K_{t-1} ∩ K_t| / |K_t| = floor(rho*k)/k exactly.  For T > 1 query
    tokens, query t>0 repeats the construction from query t-1's set with
    ratio rho_q (restricted to its own visible range)."""

    def __init__(self, seed, ctx_len, T, k, rho, zipf_s=1.1, rho_q=0.9, device="cpu"):
        self.g = _gen(seed + 32452843, device)
        self.device = device
        self.ctx_len = ctx_len.to(device=device, dtype=torch.int64)
        self.B = int(ctx_len.numel())
        self.T, self.k, self.rho, self.rho_q, self.s = T, k, rho, rho_q, zipf_s
        self.Lmax = int(self.ctx_len.max().item())
        self.prev = None

    def _logw(self, vis):
        pos = torch.arange(self.Lmax, device=self.device).unsqueeze(0)
        r = (vis.unsqueeze(1) - 1 - pos).clamp(min=0).to(torch.float32)
        lw = -self.s * torch.log(r + 1.0)
        return torch.where(pos < vis.unsqueeze(1), lw, torch.full_like(lw, float("-inf")))

    def _gumbel(self, shape):
        u = torch.rand(shape, generator=self.g, device=self.device).clamp_(1e-12, 1.0 - 1e-7)
        return -torch.log(-torch.log(u))

    def _draw(self, vis, base, keep_frac):
        """one [B,k] set: keep floor(keep_frac*k) of base (if given), rest fresh."""
        key = self._logw(vis) + self._gumbel((self.B, self.Lmax))
        if base is None:
            return key.topk(self.k, dim=1).indices
        n_keep = int(keep_frac * self.k)
        # members of base that this query can see, in random order
        r = torch.rand(base.shape, generator=self.g, device=self.device)
        r = torch.where(base < vis.unsqueeze(1), r, torch.full_like(r, -1.0))
        kept = torch.gather(base, 1, r.topk(n_keep, dim=1).indices)
        key.scatter_(1, base, float("-inf"))
        fresh = key.topk(self.k - n_keep, dim=1).indices
        return torch.cat([kept, fresh], dim=1)

    def next(self):
        """int32 [B,T,k] index sets for the next step, each in ascending order (the order in which the
        top-k kernel emits its selection)."""
        sets = []
        for t in range(self.T):
            vis = (self.ctx_len - (self.T - 1 - t)).clamp(min=0)
            if t == 0:
                base, frac = (None, 0.0) if self.prev is None else (self.prev[:, 0], self.rho)
            else:
                base, frac = sets[t - 1], self.rho_q
            sets.append(self._draw(vis, base, frac))
        cur = torch.stack(sets, dim=1)
        self.prev = cur
        return cur.sort(dim=-1).values.to(torch.int32)


PAGE_TOKENS = 64


def paged_indexer_cache(seed, key, ctx_len, n_spare_pages=3, scale_exp=(-6, 2), pow2=False, device="cpu"):
    """Scatter flat index keys [B,Lmax,Di] (uint8) into a paged pool: pages of 64 keys followed by 64
    float32 scales, placed in a seeded random order among `n_spare_pages` unused pages (filled with
    0xFF keys and NaN scales, so reading a wrong page shows).  Only pages that hold visible tokens are
    mapped; the rest of the block table is -1.  Scales are positive: 2^e * m with e uniform in
    scale_exp and m uniform in [1,2) (m = 1 when pow2).  Returns (pages uint8 [n_pages, 64*(Di+4)],
    block_table int32 [B, Lmax/64], scales float32 [B,Lmax])."""
    g = _gen(seed + 7919, "cpu")
    B, Lmax, Di = key.shape
    assert Lmax % PAGE_TOKENS == 0
    npp = Lmax // PAGE_TOKENS
    lens = ctx_len.to("cpu", torch.int64)
    used = [(int(lens[b]) + PAGE_TOKENS - 1) // PAGE_TOKENS for b in range(B)]
    n_pages = sum(used) + n_spare_pages
    perm = torch.randperm(n_pages, generator=g)
    e = torch.randint(scale_exp[0], scale_exp[1] + 1, (B, Lmax), generator=g).to(torch.float32)
    m = torch.ones((B, Lmax)) if pow2 else 1.0 + torch.rand((B, Lmax), generator=g)
    scales = (torch.pow(torch.tensor(2.0), e) * m).to(torch.float32)
    pages = torch.full((n_pages, PAGE_TOKENS * (Di + 4)), 0xFF, dtype=torch.uint8)
    pages[:, PAGE_TOKENS * Di:] = torch.tensor([float("nan")] * PAGE_TOKENS, dtype=torch.float32).view(torch.uint8)
    table = torch.full((B, npp), -1, dtype=torch.int32)
    kcpu = key.to("cpu")
    nxt = 0
    for b in range(B):
        for pg in range(used[b]):
            pid = int(perm[nxt]); nxt += 1
            table[b, pg] = pid
            pages[pid, : PAGE_TOKENS * Di] = kcpu[b, pg * PAGE_TOKENS:(pg + 1) * PAGE_TOKENS].reshape(-1)
            pages[pid, PAGE_TOKENS * Di:] = scales[b, pg * PAGE_TOKENS:(pg + 1) * PAGE_TOKENS].contiguous().view(torch.uint8)
    return pages.to(device), table.to(device), scales.to(device)
