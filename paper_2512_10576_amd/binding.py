"""Thin ctypes binding over libess.so (see include/ess.h).

Argument marshalling only: every function takes torch tensors that already
live where the C ABI expects them (device memory, or pinned host memory for
the host pool), checks dtype / contiguity, and passes raw pointers plus the
current HIP stream.  No computation happens here and there is no fallback:
if the library has not been built, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libess.so")

ESS_OK = 0
ESS_ERR_INVALID_ARG, ESS_ERR_UNSUPPORTED, ESS_ERR_CAPACITY, ESS_ERR_NOMEM, ESS_ERR_HIP = -1, -2, -3, -4, -5
ESS_ERR_INTERNAL = -6
ESS_FMT_BF16, ESS_FMT_FP8 = 0, 1
ESS_FLAG_SERIAL = 1
ESS_FLAG_DBA = 2
ESS_FLAG_AUTO = 4
ESS_FLAG_DENSE_SCORES = 8
ESS_FLAG_FUSED_SELECT = 16


class EssConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("max_batch", C.c_int32), ("max_q_tokens", C.c_int32),
                ("max_ctx", C.c_int32), ("idx_heads", C.c_int32), ("idx_dim", C.c_int32), ("topk", C.c_int32),
                ("attn_heads", C.c_int32), ("latent_fmt", C.c_int32), ("row_stride", C.c_int32),
                ("slots_per_seq", C.c_int32), ("sm_scale", C.c_float), ("flags", C.c_uint32)]


class EssCache(C.Structure):
    _fields_ = [("slot_pool", C.c_void_p), ("host_pool_dev", C.c_void_p), ("slot_of", C.c_void_p),
                ("token_of", C.c_void_p), ("stamp", C.c_void_p)]


class EssStepArgs(C.Structure):
    _fields_ = [("q_idx_fp8", C.c_void_p), ("w", C.c_void_p), ("key_fp8", C.c_void_p), ("ctx_len", C.c_void_p),
                ("q_bf16", C.c_void_p), ("topk_override", C.c_void_p), ("B", C.c_int32), ("T", C.c_int32),
                ("step", C.c_uint32), ("idx_out", C.c_void_p), ("out_bf16", C.c_void_p), ("lse", C.c_void_p),
                ("miss_count", C.c_void_p), ("block_table", C.c_void_p), ("n_pages", C.c_int32),
                ("reserved", C.c_int32)]


class EssStats(C.Structure):
    _fields_ = [("steps", C.c_uint64), ("selected", C.c_uint64), ("misses", C.c_uint64),
                ("bytes_filled", C.c_uint64)]


class EssError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libess error %d: %s" % (code, text))
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Load libess.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libess.so is not built: run `python -m paper_2512_10576_amd.build`")
    lib = C.CDLL(LIB_PATH, mode=C.RTLD_GLOBAL)
    vp, i32, u32 = C.c_void_p, C.c_int32, C.c_uint32
    sigs = {
        "ess_create": [C.POINTER(EssConfig), C.POINTER(vp)],
        "ess_destroy": [vp],
        "ess_workspace_bytes": [C.POINTER(EssConfig), C.POINTER(C.c_size_t)],
        "ess_cache_reset": [vp, C.POINTER(EssCache), i32, vp],
        "ess_cache_admit": [vp, C.POINTER(EssCache), vp, i32, i32, u32, vp],
        "ess_index_score": [vp, vp, vp, vp, vp, i32, i32, vp, vp],
        "ess_topk": [vp, vp, vp, i32, i32, vp, vp],
        "ess_topk_static": [vp, vp, i32, i32, i32, i32, vp, vp],
        "ess_gather_latent": [vp, C.POINTER(EssCache), vp, vp, i32, i32, u32, vp, vp, vp, vp],
        "ess_sparse_mla_decode": [vp, vp, vp, vp, i32, i32, vp, vp, vp],
        "ess_decode_step": [vp, C.POINTER(EssCache), C.POINTER(EssStepArgs), vp],
        "ess_get_stats": [vp, C.POINTER(EssStats), vp],
        "ess_get_seq_stats": [vp, i32, vp, vp],
        "ess_reset_stats": [vp, vp],
        "ess_profile_enable": [vp, i32],
        "ess_profile_select": [vp, u32, i32],
        "ess_calib_copy": [vp, vp, C.c_size_t, vp],
        "ess_calib_read": [vp, C.c_size_t, vp, vp],
        "ess_append": [vp, C.POINTER(EssCache), vp, vp, vp, vp, i32, i32, u32, vp, vp, vp, i32, vp],
        "ess_index_score_paged": [vp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp],
        "ess_index_topk": [vp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp],
        "ess_profile_intervals": [vp, i32, vp, vp, i32, vp],
        "ess_set_overlap_threshold": [vp, i32],
        "ess_last_overlap": [vp, C.POINTER(i32)],
        "ess_last_confined": [vp, C.POINTER(i32)],
        "ess_selfcheck_inject": [vp, i32],
        "ess_debug_ticket_grid": [vp, i32],
        "ess_calib_memcpy_rows": [vp, vp, vp, C.c_int64, i32, i32, vp],
        "ess_profile_read": [vp, C.POINTER(C.c_float), C.POINTER(i32)],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.ess_last_error.argtypes = []
    lib.ess_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc):
    if rc != ESS_OK:
        raise EssError(rc, load().ess_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None, device="cuda", optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError("tensor required")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if device == "cuda" and not t.is_cuda:
        raise ValueError("tensor must be in device memory")
    if device == "pinned" and not (t.is_pinned() or t.is_cuda):
        raise ValueError("host pool must be pinned host memory")
    return C.c_void_p(t.data_ptr())


def make_config(max_batch, max_q_tokens, max_ctx, idx_heads, idx_dim, topk, attn_heads, latent_fmt=ESS_FMT_BF16,
                row_stride=None, slots_per_seq=None, sm_scale=576 ** -0.5, flags=0) -> EssConfig:
    if row_stride is None:
        row_stride = 1152 if latent_fmt == ESS_FMT_BF16 else 656
    if slots_per_seq is None:
        slots_per_seq = max_ctx
    return EssConfig(C.sizeof(EssConfig), max_batch, max_q_tokens, max_ctx, idx_heads, idx_dim, topk, attn_heads,
                     latent_fmt, row_stride, slots_per_seq, sm_scale, flags)


def workspace_bytes(cfg: EssConfig) -> int:
    out = C.c_size_t(0)
    _check(load().ess_workspace_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def calib_copy(dst, src):
    """plain copy kernel of known traffic (measurement support)"""
    _check(load().ess_calib_copy(_ptr(dst, torch.uint8), _ptr(src, torch.uint8), src.numel(), _stream()))


CALIB_READ_WGS = 4096


def calib_read(src, sink):
    """plain read kernel over `src` (uint8, a multiple of 16 bytes); sink: int32 [CALIB_READ_WGS] on the device"""
    assert sink.numel() >= CALIB_READ_WGS
    _check(load().ess_calib_read(_ptr(src, torch.uint8), src.numel(), _ptr(sink, torch.int32), _stream()))


def calib_memcpy_rows(dst, host_pool, host_rows, row_bytes, row_stride):
    """one hipMemcpyAsync per entry: pinned `host_pool` rows `host_rows` (CPU int64 tensor) -> `dst` rows 0..n-1"""
    assert host_pool.is_pinned() and host_rows.dtype == torch.int64 and not host_rows.is_cuda and host_rows.is_contiguous()
    _check(load().ess_calib_memcpy_rows(_ptr(dst, torch.uint8), C.c_void_p(host_pool.data_ptr()),
                                        C.c_void_p(host_rows.data_ptr()), host_rows.numel(), row_bytes, row_stride,
                                        _stream()))


def topk_static(score, ctx_len, idx):
    """ess_topk without a context and without any allocation: score [B,T,max_ctx], idx [B,T,k]"""
    B, T, L = score.shape
    _check(load().ess_topk_static(_ptr(score, torch.float32), _ptr(ctx_len, torch.int32), B, T, L, idx.shape[2],
                                  _ptr(idx, torch.int32), _stream()))


class Cache:
    """Caller-owned Sparse Memory Pool state of one layer (tensors stay alive here)."""

    def __init__(self, slot_pool, slot_of, token_of, stamp, host_pool=None):
        self.slot_pool, self.slot_of, self.token_of, self.stamp, self.host_pool = slot_pool, slot_of, token_of, stamp, host_pool
        self.c = EssCache(_ptr(slot_pool, torch.uint8), _ptr(host_pool, torch.uint8, "pinned", optional=True),
                          _ptr(slot_of, torch.int32), _ptr(token_of, torch.int32), _ptr(stamp, torch.int32))

    @staticmethod
    def allocate(cfg: EssConfig, B, host_pool=None, slot_pool=None, device="cuda"):
        S, L = cfg.slots_per_seq, cfg.max_ctx
        if slot_pool is None:
            slot_pool = torch.zeros((B, S, cfg.row_stride), dtype=torch.uint8, device=device)
        return Cache(slot_pool, torch.empty((B, L), dtype=torch.int32, device=device),
                     torch.empty((B, S), dtype=torch.int32, device=device),
                     torch.empty((B, S), dtype=torch.int32, device=device), host_pool)


class Context:
    """Owns one ess_ctx.  Methods carry the names of the C entry points."""

    def __init__(self, cfg: EssConfig):
        self.lib = load()
        self.cfg = cfg
        h = C.c_void_p()
        _check(self.lib.ess_create(C.byref(cfg), C.byref(h)))
        self.h = h

    def close(self):
        if self.h:
            self.lib.ess_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def cache_reset(self, cache: Cache, B):
        _check(self.lib.ess_cache_reset(self.h, C.byref(cache.c), B, _stream()))

    def cache_admit(self, cache: Cache, tok, step):
        B, n = tok.shape
        _check(self.lib.ess_cache_admit(self.h, C.byref(cache.c), _ptr(tok, torch.int32), B, n, step, _stream()))

    def index_score(self, q_idx_fp8, w, key_fp8, ctx_len, score):
        B, T = q_idx_fp8.shape[:2]
        _check(self.lib.ess_index_score(self.h, _ptr(q_idx_fp8, torch.uint8), _ptr(w, torch.float32),
                                        _ptr(key_fp8, torch.uint8), _ptr(ctx_len, torch.int32), B, T,
                                        _ptr(score, torch.float32), _stream()))

    def topk(self, score, ctx_len, idx):
        B, T = score.shape[:2]
        _check(self.lib.ess_topk(self.h, _ptr(score, torch.float32), _ptr(ctx_len, torch.int32), B, T,
                                 _ptr(idx, torch.int32), _stream()))

    def gather_latent(self, cache: Cache, idx, ctx_len, step, slot_idx, rows_out=None, miss_count=None):
        B, T = idx.shape[:2]
        _check(self.lib.ess_gather_latent(self.h, C.byref(cache.c), _ptr(idx, torch.int32),
                                          _ptr(ctx_len, torch.int32), B, T, step, _ptr(slot_idx, torch.int32),
                                          _ptr(rows_out, torch.uint8, optional=True),
                                          _ptr(miss_count, torch.int32, optional=True), _stream()))

    def sparse_mla_decode(self, q_bf16, slot_pool, slot_idx, out_bf16, lse=None):
        B, T = q_bf16.shape[:2]
        _check(self.lib.ess_sparse_mla_decode(self.h, _ptr(q_bf16, torch.bfloat16), _ptr(slot_pool, torch.uint8),
                                              _ptr(slot_idx, torch.int32), B, T, _ptr(out_bf16, torch.bfloat16),
                                              _ptr(lse, torch.float32, optional=True), _stream()))

    def decode_step(self, cache: Cache, q_idx_fp8, w, key_fp8, ctx_len, q_bf16, step, idx_out, out_bf16, lse=None,
                    miss_count=None, topk_override=None, block_table=None):
        B, T = q_idx_fp8.shape[:2]
        a = EssStepArgs(_ptr(q_idx_fp8, torch.uint8), _ptr(w, torch.float32), _ptr(key_fp8, torch.uint8),
                        _ptr(ctx_len, torch.int32), _ptr(q_bf16, torch.bfloat16),
                        _ptr(topk_override, torch.int32, optional=True), B, T, step, _ptr(idx_out, torch.int32),
                        _ptr(out_bf16, torch.bfloat16), _ptr(lse, torch.float32, optional=True),
                        _ptr(miss_count, torch.int32, optional=True), _ptr(block_table, torch.int32, optional=True),
                        key_fp8.shape[0] if block_table is not None else 0, 0)
        _check(self.lib.ess_decode_step(self.h, C.byref(cache.c), C.byref(a), _stream()))

    def append(self, cache: Cache, new_key_fp8, new_rows, key_fp8, ctx_len, step, placed=None, new_key_scale=None,
               block_table=None):
        """write the step's new entries into the Indexer-Cache (flat, or paged with block_table and
        new_key_scale), the host pool and the slot pool; ctx_len grows"""
        B, T = new_key_fp8.shape[:2]
        n_pages = key_fp8.shape[0] if block_table is not None else 0
        _check(self.lib.ess_append(self.h, C.byref(cache.c), _ptr(new_key_fp8, torch.uint8), _ptr(new_rows, torch.uint8),
                                   _ptr(key_fp8, torch.uint8), _ptr(ctx_len, torch.int32), B, T, step,
                                   _ptr(placed, torch.int32, optional=True),
                                   _ptr(new_key_scale, torch.float32, optional=True),
                                   _ptr(block_table, torch.int32, optional=True), n_pages, _stream()))

    def index_topk(self, q_idx_fp8, w, key_fp8, ctx_len, idx, block_table=None):
        """key_fp8: [B,Lmax,Di], or the page pool when block_table is given"""
        B, T = q_idx_fp8.shape[:2]
        _check(self.lib.ess_index_topk(self.h, _ptr(q_idx_fp8, torch.uint8), _ptr(w, torch.float32), _ptr(key_fp8, torch.uint8),
                                       _ptr(block_table, torch.int32) if block_table is not None else None,
                                       key_fp8.shape[0] if block_table is not None else 0,
                                       _ptr(ctx_len, torch.int32), B, T, _ptr(idx, torch.int32), _stream()))

    def index_score_paged(self, q_idx_fp8, w, key_pages, block_table, ctx_len, score):
        B, T = q_idx_fp8.shape[:2]
        _check(self.lib.ess_index_score_paged(self.h, _ptr(q_idx_fp8, torch.uint8), _ptr(w, torch.float32),
                                              _ptr(key_pages, torch.uint8), _ptr(block_table, torch.int32),
                                              key_pages.shape[0], _ptr(ctx_len, torch.int32), B, T,
                                              _ptr(score, torch.float32), _stream()))

    def set_overlap_threshold(self, misses_per_seq):
        _check(self.lib.ess_set_overlap_threshold(self.h, misses_per_seq))

    def last_overlap(self) -> int:
        """schedule of the latest decode_step: 0 DA, 1 DBA, 2 serial"""
        m = C.c_int32(-1)
        _check(self.lib.ess_last_overlap(self.h, C.byref(m)))
        return m.value

    def last_confined(self) -> int:
        """fetches of the latest decode_step that were confined to part of the XCDs (0, 1 or 2)"""
        m = C.c_int32(-1)
        _check(self.lib.ess_last_confined(self.h, C.byref(m)))
        return m.value

    def selfcheck_inject(self, extra_items: int) -> None:
        """test hook: the self-check of the next confined step expects extra_items more work items"""
        _check(self.lib.ess_selfcheck_inject(self.h, extra_items))

    def debug_ticket_grid(self, workgroups: int) -> None:
        """test hook: ticket-fed launches use exactly `workgroups` workgroups (0 = the library's own sizing)"""
        _check(self.lib.ess_debug_ticket_grid(self.h, workgroups))

    def get_stats(self) -> dict:
        s = EssStats()
        _check(self.lib.ess_get_stats(self.h, C.byref(s), _stream()))
        return dict(steps=s.steps, selected=s.selected, misses=s.misses, bytes_filled=s.bytes_filled)

    def get_seq_stats(self, B: int) -> list:
        """per sequence: dict(steps, selected, misses, bytes_filled)"""
        arr = (EssStats * B)()
        _check(self.lib.ess_get_seq_stats(self.h, B, arr, _stream()))
        return [dict(steps=s.steps, selected=s.selected, misses=s.misses, bytes_filled=s.bytes_filled) for s in arr]

    def profile_enable(self, max_steps, stage_mask=0x3F, every=1):
        self._prof_cap = max_steps
        _check(self.lib.ess_profile_select(self.h, stage_mask, every))
        _check(self.lib.ess_profile_enable(self.h, max_steps))

    def profile_intervals(self, step):
        """[(milliseconds, stage or -1), ...]: the intervals of recorded step `step` on the caller's stream, in order;
        call before profile_read"""
        ms = (C.c_float * 64)()
        st = (C.c_int32 * 64)()
        n = C.c_int32(0)
        _check(self.lib.ess_profile_intervals(self.h, step, ms, st, 64, C.byref(n)))
        return [(ms[i], st[i]) for i in range(n.value)]

    def profile_read(self):
        """list of per-step [index_score, topk, bookkeeping, attn0, attn1+merge, fetch] milliseconds"""
        buf = (C.c_float * (self._prof_cap * 6))()
        n = C.c_int32(0)
        _check(self.lib.ess_profile_read(self.h, buf, C.byref(n)))
        return [[buf[s * 6 + i] for i in range(6)] for s in range(n.value)]

    def reset_stats(self):
        _check(self.lib.ess_reset_stats(self.h, _stream()))
