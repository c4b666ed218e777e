"""CPU oracle for the ESS decode-step hot path (test infrastructure only).

This module is the slow, plain definition of what the HIP library computes.
It is *test infrastructure*: only `tests/`, `__graft_entry__.smoke()` and the
`cpu_baseline` leg of `bench.py` may import it.  It shares no code, table or
helper with the HIP path and never imports it.

What it follows (ESS paper, arXiv 2512.10576):

  * Sec. 3 (ESS System Design): per layer and step the Indexer-Cache scores
    every Latent-Cache entry and the top 2,048 entries are selected; the
    Indexer-Cache stays on the GPU, the Latent-Cache is offloaded.
  * Sec. 2.2, Eq. (1): Intra-Layer Similarity r_t = |K_{t-1} ∩ K_t| / |K_t|.
  * Sec. 3.2 (LRU-Based Cache Eviction and Admission, LRU-Warmup): the GPU
    side Sparse Memory Pool is updated with an LRU policy, one entry being
    the swap unit (Sec. 3.1).
  * Sec. 3.1 (FlashTrans): missed entries are fetched from the CPU-side
    Total Memory Pool, which always holds every entry (Sec. 3.3: new
    entries are written back to it), so eviction needs no write-back.
  * Sec. 3.3 (DA Overlap): SparseMLA is split in Attn0 (resident entries)
    and Attn1 (fetched entries) and the two results are merged.

The paper does not print the indexer formula, the tie rule of the top-k, the
LRU granularity or the merge rule; the readings taken here are stated in the
docstring of each function and collected in the design notes of the
repository.

Pins (see tests/test_oracle_*.py): every function below is pinned to
something other than itself -- int64 brute force, exhaustive Python sort,
torch's scaled_dot_product_attention on the CPU with an additive mask,
torch's float8_e4m3fn / bfloat16 casts, a textbook OrderedDict LRU in the
one-access-per-step special case, closed forms and invariants; the append
against a hand-worked example (tests/golden), the same OrderedDict LRU, and
a decode loop over an appended context against the same loop over a context
built whole.  The LRU
bookkeeping for several accesses per step has no counterpart printed in the
paper: beyond the special case and the invariants it is "parity unpinned"
against the paper.

All floating point is float64 unless the value is exactly representable in
less (index scores on integer-valued inputs).
"""
from __future__ import annotations

import numpy as np

LATENT_DIM = 512   # value / compressed-KV part of one Latent-Cache entry
ROPE_DIM = 64      # rotary part of one Latent-Cache entry
ROW_DIM = LATENT_DIM + ROPE_DIM
FMT_BF16 = 0       # 576 x bf16                       = 1152 bytes
FMT_FP8 = 1        # 512 x e4m3 + 4 x bf16 scale + 64 x bf16 rope = 648 bytes
FP8_GROUP = 128    # elements that share one scale in FMT_FP8
NEG_INF = -np.inf


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------
def e4m3fn_table() -> np.ndarray:
    """All 256 values of OCP FP8 E4M3 (the "fn" flavour: no infinities, one
    NaN mantissa pattern per sign), built from the format definition:
    1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent field
    0 is subnormal (value = mantissa/8 * 2^-6); exponent 15 with mantissa 7
    is NaN; every other pattern is (1 + mantissa/8) * 2^(exponent - 7)."""
    out = np.empty(256, dtype=np.float64)
    for byte in range(256):
        sign = -1.0 if byte & 0x80 else 1.0
        expo = (byte >> 3) & 0xF
        mant = byte & 0x7
        if expo == 0xF and mant == 0x7:
            val = np.nan
        elif expo == 0:
            val = sign * (mant / 8.0) * 2.0 ** (-6)
        else:
            val = sign * (1.0 + mant / 8.0) * 2.0 ** (expo - 7)
        out[byte] = val
    return out


_E4M3 = e4m3fn_table()


def decode_e4m3(byte_array: np.ndarray) -> np.ndarray:
    """uint8 array -> float64 values of the E4M3 patterns."""
    return _E4M3[np.asarray(byte_array, dtype=np.uint8)]


def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bfloat16 -> float64.  bfloat16 is the upper
    half of an IEEE binary32, so the value is the binary32 whose top 16 bits
    are the pattern and whose low 16 bits are zero."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def decode_rows(row_bytes: np.ndarray, fmt: int) -> np.ndarray:
    """Latent-Cache entries as bytes [..., stride] -> float64 [..., 576].

    FMT_BF16: 576 little-endian bfloat16 (512 latent then 64 rope).
    FMT_FP8 : bytes [0,512) E4M3 latent, [512,520) four bfloat16 scales (one
    per 128 latent elements), [520,648) 64 bfloat16 rope values; element i of
    the latent is e4m3(byte_i) * scale[i // 128].  Bytes past the format's
    length (stride padding) are ignored."""
    rb = np.ascontiguousarray(row_bytes, dtype=np.uint8)
    lead = rb.shape[:-1]
    if fmt == FMT_BF16:
        raw = np.ascontiguousarray(rb[..., : ROW_DIM * 2])
        return decode_bf16(raw.view(np.uint16).reshape(*lead, ROW_DIM))
    if fmt == FMT_FP8:
        lat = decode_e4m3(rb[..., :LATENT_DIM])
        sc = decode_bf16(np.ascontiguousarray(rb[..., 512:520]).view(np.uint16).reshape(*lead, 4))
        lat = lat * np.repeat(sc, FP8_GROUP, axis=-1)
        rope = decode_bf16(np.ascontiguousarray(rb[..., 520:648]).view(np.uint16).reshape(*lead, ROPE_DIM))
        return np.concatenate([lat, rope], axis=-1)
    raise ValueError("unknown latent format")


# --------------------------------------------------------------------------
# stage 1: index score
# --------------------------------------------------------------------------
def visible(ctx_len: np.ndarray, T: int, t: int) -> np.ndarray:
    """Number of cached positions query token t (of T per sequence) may see.
    Reading for multi-token decode (the paper's MTP setting, Table 1): the
    cache already holds the T new tokens at the last T positions, and query t
    sees itself and everything before: vis = ctx_len - (T - 1 - t)."""
    return np.maximum(np.asarray(ctx_len, dtype=np.int64) - (T - 1 - t), 0)


def index_score(q_u8, w, key_u8, ctx_len) -> np.ndarray:
    """Importance of every cached token (Sec. 3: the Indexer-Cache "computes
    the importance of each Latent-Cache entry"):

        score[b,t,s] = sum_j w[b,t,j] * max(0, sum_d q[b,t,j,d] * key[b,s,d])

    for s < vis(b,t); -inf elsewhere.  One key per token is shared by all
    indexer heads.  q_u8 [B,T,Hi,Di] and key_u8 [B,Lmax,Di] are E4M3 bytes,
    w [B,T,Hi] float32.  Computed in float64 (exact for the integer-valued
    test inputs, whose partial sums stay far below 2^53) and returned as
    float32, which is exact whenever 2^24 bounds the result in units of the
    input grid."""
    q = decode_e4m3(q_u8)
    key = decode_e4m3(key_u8)
    w64 = np.asarray(w, dtype=np.float64)
    B, T, Hi, Di = q.shape
    Lmax = key.shape[1]
    out = np.full((B, T, Lmax), NEG_INF, dtype=np.float32)
    for b in range(B):
        for t in range(T):
            vis = int(visible(ctx_len, T, t)[b])
            if vis <= 0:
                continue
            dots = key[b, :vis] @ q[b, t].T              # [vis, Hi]
            act = np.maximum(dots, 0.0)
            out[b, t, :vis] = (act @ w64[b, t]).astype(np.float32)
    return out


PAGE_TOKENS = 64   # tokens per page of the paged Indexer-Cache


def page_bytes(Di: int) -> int:
    """One page: PAGE_TOKENS keys of Di E4M3 bytes, then PAGE_TOKENS float32
    scales (little endian), one per key: (Di + 4) bytes per token, the 132
    bytes per token behind the paper's 16.8 % = 132 / (132 + 656) (Sec. 3)."""
    return PAGE_TOKENS * (Di + 4)


def paged_keys(key_pages, block_table, b: int, n_tok: int, Di: int):
    """Keys and scales of the first n_tok tokens of sequence b, through its
    block table: token s lives in page block_table[b, s // 64], row s % 64.
    key_pages uint8 [n_pages, page_bytes(Di)].  Returns (uint8 [n_tok,Di],
    float32 [n_tok])."""
    keys = np.zeros((n_tok, Di), dtype=np.uint8)
    scales = np.zeros(n_tok, dtype=np.float32)
    for s in range(n_tok):
        page = key_pages[int(block_table[b, s // PAGE_TOKENS])]
        r = s % PAGE_TOKENS
        keys[s] = page[r * Di:(r + 1) * Di]
        scales[s] = page[PAGE_TOKENS * Di + 4 * r: PAGE_TOKENS * Di + 4 * r + 4].view(np.float32)[0]
    return keys, scales


def index_score_paged(q_u8, w, key_pages, block_table, ctx_len) -> np.ndarray:
    """Index score over a paged Indexer-Cache with one scale per key (the
    layout behind the paper's `paged_mqa_logits` and its 132-byte Indexer
    entries, Sec. 3 / 3.3).  The stored key of token s stands for
    scale_s * key_s, scale_s > 0, so

        score[b,t,s] = sum_j w_j * max(0, q_j . (scale_s * key_s))
                     = scale_s * sum_j w_j * max(0, q_j . key_s).

    Reading (the paper prints neither form): the second form is the
    definition, evaluated as float32(sum) * float32(scale) rounded once to
    float32 -- with integer-valued inputs the sum is exact, so the result does
    not depend on the summation order.  Positions s >= vis(b,t): -inf.
    Returns float32 [B,T,Lmax] with Lmax = 64 * block_table.shape[1]."""
    q = decode_e4m3(q_u8)
    w64 = np.asarray(w, dtype=np.float64)
    B, T, Hi, Di = q.shape
    Lmax = PAGE_TOKENS * block_table.shape[1]
    out = np.full((B, T, Lmax), NEG_INF, dtype=np.float32)
    for b in range(B):
        n_tok = int(min(max(int(ctx_len[b]), 0), Lmax))
        kb, sc = paged_keys(key_pages, block_table, b, n_tok, Di)
        key = decode_e4m3(kb)
        for t in range(T):
            vis = int(visible(ctx_len, T, t)[b])
            if vis <= 0:
                continue
            act = np.maximum(key[:vis] @ q[b, t].T, 0.0)
            base = (act @ w64[b, t]).astype(np.float32)
            out[b, t, :vis] = base * sc[:vis]              # float32 * float32, one rounding
    return out


# --------------------------------------------------------------------------
# stage 2: top-k
# --------------------------------------------------------------------------
def topk(score, ctx_len, k: int) -> np.ndarray:
    """Indices of the k most important visible tokens per query (Sec. 3:
    "selecting the top 2,048 critical entries").

    The paper does not say how equal scores are ordered; reading: the total
    order is (score descending, index ascending), so the result is the first
    min(k, vis) visible positions under that order, listed in that order;
    the remaining entries are -1.  NaN scores rank as -inf.  +0.0 and -0.0
    are equal.  Returns int32 [B,T,k]."""
    sc = np.asarray(score, dtype=np.float32)
    B, T, Lmax = sc.shape
    out = np.full((B, T, k), -1, dtype=np.int32)
    for b in range(B):
        for t in range(T):
            vis = int(min(visible(ctx_len, T, t)[b], Lmax))
            if vis <= 0:
                continue
            row = sc[b, t, :vis].astype(np.float64)
            row = np.where(np.isnan(row), NEG_INF, row)
            order = np.argsort(-row, kind="stable")      # stable: ties keep index order
            n = min(k, vis)
            out[b, t, :n] = order[:n]
    return out


def intra_layer_similarity(prev_idx, cur_idx) -> float:
    """Eq. (1): |K_{t-1} ∩ K_t| / |K_t| for two index lists (-1 = padding)."""
    a = set(int(x) for x in np.asarray(prev_idx).ravel() if x >= 0)
    c = set(int(x) for x in np.asarray(cur_idx).ravel() if x >= 0)
    return len(a & c) / max(len(c), 1)


# --------------------------------------------------------------------------
# stages 3 + 5: Sparse Memory Pool (slot cache) with step-granular LRU
# --------------------------------------------------------------------------
class SlotCache:
    """GPU-side Sparse Memory Pool of one layer (Sec. 3.2), one fixed-size
    pool of S slots per sequence, an entry (one token's Latent-Cache row)
    being the swap unit (Sec. 3.1).

    The paper says "LRU-based"; everything finer is a reading.  Per sequence
    and step `step_no` (numbered from 1, strictly increasing):

      1. R = the set of distinct valid indices selected by the T queries.
      2. hits = members of R that are resident; their slot's stamp := step_no.
      3. misses = the rest of R, in ascending token index; m = their number.
      4. victims = the m slots smallest in (stamp, slot index) among slots
         whose stamp < step_no (empty slots carry stamp 0 and so go first).
         The i-th miss takes the i-th victim.
      5. per pair: the victim's former token (if any) becomes non-resident;
         token_of[victim] = miss, slot_of[miss] = victim, stamp := step_no,
         and the row is copied from the host pool into the slot.

    Entries touched in the current step are thereby unevictable (attention
    needs all of R resident at once) and the outcome does not depend on the
    order in which the top-k lists its indices.  len(R) > S is an error.

    State (caller-visible, mirrors the library's arrays):
      slot_of  int32 [B,Lmax]  slot of a token, -1 = not resident
      token_of int32 [B,S]     token in a slot, -1 = empty
      stamp    uint32 [B,S]    step of last use, 0 = never used
    """

    def __init__(self, B: int, Lmax: int, S: int):
        self.B, self.Lmax, self.S = B, Lmax, S
        self.slot_of = np.full((B, Lmax), -1, dtype=np.int32)
        self.token_of = np.full((B, S), -1, dtype=np.int32)
        self.stamp = np.zeros((B, S), dtype=np.uint32)

    def make_resident_identity(self):
        """Fully resident mode (no offload): slot s holds token s."""
        assert self.S == self.Lmax
        ar = np.arange(self.Lmax, dtype=np.int32)
        self.slot_of[:] = ar
        self.token_of[:] = ar

    def step(self, idx, step_no: int):
        """Apply one step.  idx int32 [B,T,k] (-1 = padding).
        Returns dict with
          slot_idx  int32 [B,T,k]  slot of every selected token after the step (-1 where idx is -1)
          fresh     bool  [B,T,k]  True where the token was a miss in this step
          miss_tok  list of B int32 arrays (ascending token index)
          victims   list of B int32 arrays (slot taken by the i-th miss)
          miss_count int32 [B]"""
        idx = np.asarray(idx, dtype=np.int32)
        B, T, k = idx.shape
        assert B == self.B
        slot_idx = np.full((B, T, k), -1, dtype=np.int32)
        fresh = np.zeros((B, T, k), dtype=bool)
        miss_tok, victims = [], []
        miss_count = np.zeros(B, dtype=np.int32)
        for b in range(B):
            sel = idx[b].ravel()
            R = np.unique(sel[sel >= 0])                       # ascending, distinct
            if R.size > self.S:
                raise ValueError("selected set larger than the slot pool")
            resident = self.slot_of[b, R] >= 0
            hits = R[resident]
            self.stamp[b, self.slot_of[b, hits]] = step_no
            M = R[~resident]
            m = int(M.size)
            cand = np.nonzero(self.stamp[b] < step_no)[0]
            order = np.lexsort((cand, self.stamp[b, cand]))    # primary stamp, then slot
            V = cand[order][:m].astype(np.int32)
            assert V.size == m, "not enough evictable slots"
            for s, v in zip(M, V):
                old = self.token_of[b, v]
                if old >= 0:
                    self.slot_of[b, old] = -1
                self.token_of[b, v] = s
                self.slot_of[b, s] = v
                self.stamp[b, v] = step_no
            miss_tok.append(M.astype(np.int32))
            victims.append(V)
            miss_count[b] = m
            valid = idx[b] >= 0
            slot_idx[b][valid] = self.slot_of[b, idx[b][valid]]
            fresh[b][valid] = np.isin(idx[b][valid], M)
        return dict(slot_idx=slot_idx, fresh=fresh, miss_tok=miss_tok,
                    victims=victims, miss_count=miss_count)


def fill_slots(slot_pool, host_pool, miss_tok, victims) -> int:
    """Sec. 3.1: copy every missed entry from the CPU-side Total Memory Pool
    (host_pool uint8 [B,Lmax,stride]) into its slot of the Sparse Memory Pool
    (slot_pool uint8 [B,S,stride]); byte-for-byte.  Returns bytes moved."""
    moved = 0
    for b, (M, V) in enumerate(zip(miss_tok, victims)):
        if len(M):
            slot_pool[b, V] = host_pool[b, M]
            moved += len(M) * host_pool.shape[-1]
    return moved


def gather_rows(slot_pool, slot_idx) -> np.ndarray:
    """rows[b,t,j,:] = slot_pool[b, slot_idx[b,t,j], :]; zero rows where
    slot_idx is -1.  uint8 [B,T,k,stride]."""
    B, T, k = slot_idx.shape
    out = np.zeros((B, T, k, slot_pool.shape[-1]), dtype=np.uint8)
    for b in range(B):
        v = slot_idx[b] >= 0
        out[b][v] = slot_pool[b, slot_idx[b][v]]
    return out


# --------------------------------------------------------------------------
# stage 4: sparse MLA decode attention
# --------------------------------------------------------------------------
def sparse_mla(q_bits, slot_pool, slot_idx, fmt: int, sm_scale: float):
    """SparseMLA over the selected Latent-Cache entries (Sec. 3.3), absorbed
    form: the 576-d entry is the key, its first 512 dims are the value.

        z_s   = sm_scale * sum_{d<576} q[d] * c_s[d]       (s over selected rows)
        lse   = log sum_s exp(z_s)
        out   = sum_s exp(z_s - lse) * c_s[:512]

    q_bits uint16 [B,T,H,576] (bfloat16 patterns); slot_pool uint8
    [B,S,stride]; slot_idx int32 [B,T,k], -1 entries are skipped.
    Empty selection: out = 0, lse = -inf.  Returns (out f64 [B,T,H,512],
    lse f64 [B,T,H])."""
    q = decode_bf16(q_bits)
    B, T, H, D = q.shape
    assert D == ROW_DIM
    out = np.zeros((B, T, H, LATENT_DIM), dtype=np.float64)
    lse = np.full((B, T, H), NEG_INF, dtype=np.float64)
    for b in range(B):
        for t in range(T):
            sl = slot_idx[b, t]
            sl = sl[sl >= 0]
            if sl.size == 0:
                continue
            c = decode_rows(slot_pool[b, sl], fmt)            # [n,576]
            z = sm_scale * (q[b, t] @ c.T)                     # [H,n]
            zmax = z.max(axis=1, keepdims=True)
            e = np.exp(z - zmax)
            den = e.sum(axis=1, keepdims=True)
            lse[b, t] = (zmax + np.log(den))[:, 0]
            out[b, t] = (e / den) @ c[:, :LATENT_DIM]
    return out, lse


def merge_partials(o0, l0, o1, l1):
    """Merge of Attn0 and Attn1 (Sec. 3.3 says only that the two results are
    merged).  Reading: both are softmax-normalised over their own rows, so
    the exact combination is lse = log(e^l0 + e^l1),
    out = e^(l0-lse) * o0 + e^(l1-lse) * o1; a part with l = -inf is empty
    and contributes nothing."""
    l0 = np.asarray(l0, dtype=np.float64)
    l1 = np.asarray(l1, dtype=np.float64)
    lse = np.logaddexp(l0, l1)
    with np.errstate(invalid="ignore"):
        w0 = np.where(np.isneginf(l0), 0.0, np.exp(l0 - lse))
        w1 = np.where(np.isneginf(l1), 0.0, np.exp(l1 - lse))
    out = w0[..., None] * np.asarray(o0, dtype=np.float64) + w1[..., None] * np.asarray(o1, dtype=np.float64)
    return out, lse


# --------------------------------------------------------------------------
# append: the entries the step itself produces
# --------------------------------------------------------------------------
def append_tokens(cache: SlotCache, key_u8, host_pool, slot_pool, ctx_len,
                  new_key_u8, new_rows, step_no: int, paged=None) -> np.ndarray:
    """Sec. 3.3: after a step the newly generated entries go into the caches.
    For sequence b with L0 = ctx_len[b], the t-th of its T new tokens gets
    position p = L0 + t (tokens that would pass Lmax are dropped):

      * its index key is written into the Indexer-Cache (GPU): key[b,p] = new_key[b,t];
      * its Latent-Cache entry is written back to the CPU-side Total Memory
        Pool (the paper's D2H transfer): host_pool[b,p] = new_rows[b,t];
      * reading (the paper does not say whether the new entry also enters the
        GPU pool): it is admitted to the Sparse Memory Pool as the most
        recently used entry -- the slot smallest in (stamp, slot index) among
        slots with stamp < step_no is taken, exactly the victim rule of
        SlotCache.step; its former token becomes non-resident; the slot gets
        stamp step_no and the entry's bytes.  With no slot below step_no the
        entry simply stays non-resident (it is in the host pool);
      * fully resident mode (host_pool None, S = Lmax, slot = position):
        the entry goes to slot p;
      * ctx_len[b] = L0 + (number of tokens placed).

    Paged Indexer-Cache: paged = (key_pages, block_table, new_scale) with
    new_scale float32 [B,T]; key_u8 is then unused (None), Lmax = 64 * pages
    per sequence, and the key and its scale go to row p % 64 of page
    block_table[b, p // 64].  The caller maps pages ahead of the context; a
    token whose page is unmapped (negative id) is dropped like one past Lmax,
    and so are the tokens after it.

    All arrays are updated in place; returns int32 [B,T] with the slot each
    new token went to (-1 = dropped or not admitted)."""
    B, T, Di = new_key_u8.shape
    Lmax = key_u8.shape[1] if paged is None else PAGE_TOKENS * paged[1].shape[1]
    placed = np.full((B, T), -1, dtype=np.int32)
    for b in range(B):
        L0 = int(ctx_len[b])
        n = max(0, min(T, Lmax - L0))
        if paged is not None:
            for t in range(n):
                if paged[1][b, (L0 + t) // PAGE_TOKENS] < 0:
                    n = t
                    break
        for t in range(n):
            p = L0 + t
            if paged is None:
                key_u8[b, p] = new_key_u8[b, t]
            else:
                page = paged[0][int(paged[1][b, p // PAGE_TOKENS])]
                r = p % PAGE_TOKENS
                page[r * Di:(r + 1) * Di] = new_key_u8[b, t]
                page[PAGE_TOKENS * Di + 4 * r: PAGE_TOKENS * Di + 4 * r + 4] = \
                    np.asarray(paged[2][b, t], dtype=np.float32).reshape(1).view(np.uint8)
            if host_pool is None:
                v = p
            else:
                host_pool[b, p] = new_rows[b, t]
                cand = np.nonzero(cache.stamp[b] < step_no)[0]
                if cand.size == 0:
                    continue
                v = int(cand[np.lexsort((cand, cache.stamp[b, cand]))[0]])
            old = cache.token_of[b, v]
            if old >= 0:
                cache.slot_of[b, old] = -1
            cache.token_of[b, v] = p
            cache.slot_of[b, p] = v
            cache.stamp[b, v] = step_no
            slot_pool[b, v] = new_rows[b, t]
            placed[b, t] = v
        ctx_len[b] = L0 + n
    return placed


# --------------------------------------------------------------------------
# whole step
# --------------------------------------------------------------------------
def decode_step(q_idx_u8, w, key_u8, ctx_len, k, cache: SlotCache, slot_pool,
                host_pool, q_bits, fmt, sm_scale, step_no, topk_override=None, paged=None):
    """One layer-step: index score -> top-k -> (optional trace override) ->
    LRU bookkeeping -> miss fill -> sparse MLA.  `cache` and `slot_pool` are
    updated in place.  host_pool None means fully resident (no misses may
    occur).  Returns dict(score, idx, used_idx, slot_idx, fresh, miss_count,
    out, lse)."""
    if paged is None:
        score = index_score(q_idx_u8, w, key_u8, ctx_len)
    else:                                   # (key_pages, block_table): paged Indexer-Cache, key_u8 unused
        score = index_score_paged(q_idx_u8, w, paged[0], paged[1], ctx_len)
    idx = topk(score, ctx_len, k)
    used = idx if topk_override is None else np.asarray(topk_override, dtype=np.int32)
    bk = cache.step(used, step_no)
    if host_pool is None:
        assert int(bk["miss_count"].sum()) == 0
    else:
        fill_slots(slot_pool, host_pool, bk["miss_tok"], bk["victims"])
    out, lse = sparse_mla(q_bits, slot_pool, bk["slot_idx"], fmt, sm_scale)
    return dict(score=score, idx=idx, used_idx=used, slot_idx=bk["slot_idx"],
                fresh=bk["fresh"], miss_count=bk["miss_count"], out=out, lse=lse)
