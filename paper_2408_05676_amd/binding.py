"""ctypes marshalling for the C ABI declared in include/laser.h (same names, same arguments).

There is no fallback of any kind: if liblaser.so is missing or a call fails, LaserError is raised.
"""
from __future__ import annotations

import ctypes as C
import sys
import os

import numpy as np
import torch

MODE_RV, MODE_RV_OR_TOP1, MODE_TOPK_ONLY, MODE_TOPP_ONLY = 0, 1, 2, 3
MAX_NGRAM, MAX_DRAFT, MAX_TOPK, MAX_TREE, MAX_OWN_TEXT = 8, 63, 8, 32, 4096      # LASER_MAX_* of include/laser.h

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class LaserError(RuntimeError):
    pass


def lib_path() -> str:
    return os.path.join(_HERE, "liblaser.so")


class _ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "ffn", "vocab",
                                         "max_rows", "max_batch", "max_pos")] + \
               [("eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_void_p) for n in ("wqkv", "wo", "wgu", "wdown", "g1", "g2", "emb", "wlm", "gf")]


class _KVDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "n_heads", "head_dim", "page_size", "n_pages",
                                         "max_seqs", "max_pages_per_seq")]


def lib():
    """Load liblaser.so once and declare the prototypes."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise LaserError(f"{path} is not built; run `python -m paper_2408_05676_amd.build` "
                         "(or __graft_entry__.build()) first. There is no fallback path.")
    L = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    L.laser_last_error.restype = C.c_char_p
    L.laser_version.restype = C.c_char_p
    protos = {
        "laser_pool_build": [vp, vp, vp, i64, i32, vp, C.POINTER(vp)],
        "laser_pool_destroy": [vp],
        "laser_pool_info": [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)],
        "laser_pool_read_tokens": [vp, i64, i64, vp],
        "laser_retrieve_drafts": [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp],
        "laser_retrieve_drafts_temp": [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp],
        "laser_own_text_append": [vp, vp, i32, vp, vp, i32, i32, vp],
        "laser_model_create": [C.POINTER(_ModelDesc), vp, C.POINTER(vp)],
        "laser_model_destroy": [vp],
        "laser_kv_create": [C.POINTER(_KVDesc), vp, C.POINTER(vp)],
        "laser_kv_destroy": [vp],
        "laser_kv_seq_reserve": [vp, i32, i32, vp],
        "laser_kv_seq_release": [vp, i32, vp],
        "laser_kv_import": [vp, i32, i32, vp, vp, i32, vp],
        "laser_kv_seq_set_len": [vp, i32, i32, vp],
        "laser_kv_read_lens": [vp, vp, i32, vp, vp],
        "laser_verify_step": [vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, vp, vp, vp],
        "laser_verify_head": [vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, vp, vp, vp],
        "laser_verify_head_static": [vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, vp, vp],
        "laser_kv_commit": [vp, vp, vp, i32, vp],
        "laser_kv_commit_tree": [vp, vp, vp, vp, i32, i32, vp],
        "laser_generate": [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, C.POINTER(C.c_int), C.POINTER(C.c_float), vp],
        "laser_retrieve_tree": [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp],
        "laser_verify_tree": [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, i32, vp, vp, vp, vp, vp],
        "laser_ctx_advance": [vp, vp, vp, vp, i32, i32, i32, vp],
        "laser_profile_begin": [vp, i32],
        "laser_model_set_option": [vp, C.c_char_p, i32],
        "laser_model_status": [vp, vp, C.POINTER(C.c_int)],
        "laser_model_read_trace": [vp, vp, vp, i32, C.POINTER(C.c_int), C.POINTER(C.c_int)],
        "laser_profile_end": [vp, vp, C.POINTER(C.c_float), C.POINTER(C.c_int)],
        "laser_probe_hbm": [vp, C.c_size_t, i32, vp, C.POINTER(C.c_float), C.POINTER(C.c_float)],
        "laser_probe_mfma_f16": [vp, i32, vp, C.POINTER(C.c_float)],
        "laser_probe_launch": [i32, i32, vp, C.POINTER(C.c_float)],
        "laser_probe_exchange": [vp, C.c_size_t, i32, vp, C.POINTER(C.c_float), C.POINTER(C.c_int)],
    }
    for name, args in protos.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = C.c_int
    _LIB = L
    return L


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise LaserError(f"{what} failed with code {rc}: {lib().laser_last_error().decode()}")


def _stream(stream=None) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise LaserError(f"{name} must be a contiguous CUDA tensor of {dtype}")
    return t.data_ptr()


def _host_i32(a, name: str) -> np.ndarray:
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    if arr.ndim != 1:
        raise LaserError(f"{name} must be one-dimensional")
    return arr


class Pool:
    """laser_pool_build / laser_pool_destroy."""

    def __init__(self, tokens, seq_off, seq_key, n_max: int, stream=None):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        seq_off = np.ascontiguousarray(seq_off, dtype=np.int64)
        seq_key = np.ascontiguousarray(seq_key, dtype=np.int64)
        if seq_off.size != seq_key.size + 1:
            raise LaserError("seq_off must have n_seq + 1 entries")
        if seq_key.size and int(seq_off[-1]) != tokens.size:
            raise LaserError("seq_off[-1] must equal the number of tokens")
        self._h = C.c_void_p()
        self.n_max = n_max
        _check(lib().laser_pool_build(tokens.ctypes.data, seq_off.ctypes.data, seq_key.ctypes.data,
                                      seq_key.size, n_max, _stream(stream), C.byref(self._h)),
               "laser_pool_build")

    def info(self) -> dict:
        v = [C.c_int64() for _ in range(4)]
        _check(lib().laser_pool_info(self._h, *[C.byref(x) for x in v]), "laser_pool_info")
        return dict(zip(("n_tokens", "n_keys", "n_index_entries", "device_bytes"), (x.value for x in v)))

    def read_tokens(self, start: int, count: int) -> np.ndarray:
        out = np.empty(count, dtype=np.int32)
        _check(lib().laser_pool_read_tokens(self._h, start, count, out.ctypes.data), "laser_pool_read_tokens")
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().laser_pool_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        # at interpreter shutdown the HIP runtime may already be gone; the process frees everything
        if not sys.is_finalizing():
            self.close()


def retrieve_drafts(pool: Pool, keys: torch.Tensor, ctx_tail: torch.Tensor, n_min: int, n_max: int,
                    K: int, min_tokens: int = 1, out=None, stream=None):
    """laser_retrieve_drafts. Returns (drafts [B][K], draft_len [B], match_n [B], pool_index [B])."""
    B = keys.shape[0]
    if ctx_tail.shape != (B, n_max):
        raise LaserError("ctx_tail must be [B][n_max]")
    dev = keys.device
    if out is None:
        out = (torch.empty((B, K), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int64, device=dev))
    drafts, dl, mn, pi = out
    _check(lib().laser_retrieve_drafts(pool._h, _dev(keys, torch.int64, "keys"), _dev(ctx_tail, torch.int32, "ctx_tail"),
                                       B, n_min, n_max, K, min_tokens,
                                       _dev(drafts, torch.int32, "drafts") if K > 0 else None,
                                       _dev(dl, torch.int32, "draft_len"), _dev(mn, torch.int32, "match_n"),
                                       _dev(pi, torch.int64, "pool_index"), _stream(stream)),
           "laser_retrieve_drafts")
    return drafts, dl, mn, pi


def retrieve_drafts_temp(pool: Pool, keys: torch.Tensor, ctx_tail: torch.Tensor, own_tokens: torch.Tensor,
                         own_len: torch.Tensor, n_min: int, n_max: int, K: int, min_tokens: int = 1, out=None, stream=None):
    """laser_retrieve_drafts_temp: the lookup with each sequence's own text [B][own_cap] as a temporary branch."""
    B = keys.shape[0]
    if ctx_tail.shape != (B, n_max):
        raise LaserError("ctx_tail must be [B][n_max]")
    if own_tokens.dim() != 2 or own_tokens.shape[0] != B or own_len.shape != (B,):
        raise LaserError("own_tokens must be [B][own_cap] and own_len [B]")
    dev = keys.device
    if out is None:
        out = (torch.empty((B, K), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int64, device=dev))
    drafts, dl, mn, pi = out
    _check(lib().laser_retrieve_drafts_temp(pool._h, _dev(keys, torch.int64, "keys"), _dev(ctx_tail, torch.int32, "ctx_tail"),
                                            _dev(own_tokens, torch.int32, "own_tokens"), _dev(own_len, torch.int32, "own_len"),
                                            own_tokens.shape[1], B, n_min, n_max, K, min_tokens,
                                            _dev(drafts, torch.int32, "drafts") if K > 0 else None,
                                            _dev(dl, torch.int32, "draft_len"), _dev(mn, torch.int32, "match_n"),
                                            _dev(pi, torch.int64, "pool_index"), _stream(stream)),
           "laser_retrieve_drafts_temp")
    return drafts, dl, mn, pi


def own_text_append(own_tokens: torch.Tensor, own_len: torch.Tensor, out_tokens: torch.Tensor, accept_len: torch.Tensor,
                    stream=None):
    """laser_own_text_append."""
    B, cap = own_tokens.shape
    K = out_tokens.shape[1] - 1
    _check(lib().laser_own_text_append(_dev(own_tokens, torch.int32, "own_tokens"), _dev(own_len, torch.int32, "own_len"), cap,
                                       _dev(out_tokens, torch.int32, "out_tokens"), _dev(accept_len, torch.int32, "accept_len"),
                                       B, K, _stream(stream)), "laser_own_text_append")


class Model:
    """laser_model_create / laser_model_destroy. `weights` maps the names of laser_model_desc to
    CUDA tensors (bf16 matrices stacked over layers, float32 gains); they are borrowed, and kept
    alive by this object."""

    def __init__(self, n_layers, d_model, n_heads, ffn, vocab, weights: dict, max_rows: int, max_batch: int,
                 max_pos: int, eps: float = 1e-6, rope_base: float = 10000.0, stream=None):
        self.n_layers, self.d, self.n_heads, self.ffn, self.vocab = n_layers, d_model, n_heads, ffn, vocab
        self.max_rows, self.max_batch = max_rows, max_batch
        self._keep = dict(weights)
        d = _ModelDesc(n_layers, d_model, n_heads, ffn, vocab, max_rows, max_batch, max_pos, eps, rope_base)
        for name in ("wqkv", "wo", "wgu", "wdown", "emb", "wlm"):
            t = weights.get(name)
            if t is None:
                if n_layers == 0 and name != "wlm":
                    continue
                raise LaserError(f"missing weight {name}")
            setattr(d, name, _dev(t, torch.bfloat16, name))
        for name in ("g1", "g2", "gf"):
            t = weights.get(name)
            if t is None:
                if n_layers == 0:
                    continue
                raise LaserError(f"missing weight {name}")
            setattr(d, name, _dev(t, torch.float32, name))
        self._h = C.c_void_p()
        _check(lib().laser_model_create(C.byref(d), _stream(stream), C.byref(self._h)), "laser_model_create")

    def set_option(self, name: str, value: int):
        _check(lib().laser_model_set_option(self._h, name.encode(), value), "laser_model_set_option")

    def aborted(self, stream=None) -> bool:
        v = C.c_int()
        _check(lib().laser_model_status(self._h, _stream(stream), C.byref(v)), "laser_model_status")
        return bool(v.value)

    def read_trace(self, stream=None) -> np.ndarray:
        """int64[nwg][cap] wall-clock stamps (100 MHz) of the last traced persistent-kernel launch."""
        buf = np.zeros(1 << 20, dtype=np.int64)
        nwg, cap = C.c_int(), C.c_int()
        _check(lib().laser_model_read_trace(self._h, _stream(stream), buf.ctypes.data, buf.size, C.byref(nwg), C.byref(cap)),
               "laser_model_read_trace")
        return buf[:nwg.value * cap.value].reshape(nwg.value, cap.value)

    def profile_begin(self, max_records: int):
        _check(lib().laser_profile_begin(self._h, max_records), "laser_profile_begin")

    def profile_end(self, stream=None):
        ms, n = C.c_float(), C.c_int()
        _check(lib().laser_profile_end(self._h, _stream(stream), C.byref(ms), C.byref(n)), "laser_profile_end")
        return ms.value, n.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().laser_model_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        # at interpreter shutdown the HIP runtime may already be gone; the process frees everything
        if not sys.is_finalizing():
            self.close()


class KVCache:
    """laser_kv_create and the per-slot calls."""

    def __init__(self, n_layers, n_heads, head_dim, n_pages, max_seqs, max_pages_per_seq, page_size=16,
                 stream=None):
        self.page_size = page_size
        d = _KVDesc(n_layers, n_heads, head_dim, page_size, n_pages, max_seqs, max_pages_per_seq)
        self._h = C.c_void_p()
        _check(lib().laser_kv_create(C.byref(d), _stream(stream), C.byref(self._h)), "laser_kv_create")

    def reserve(self, seq: int, n_tokens: int, stream=None):
        _check(lib().laser_kv_seq_reserve(self._h, seq, n_tokens, _stream(stream)), "laser_kv_seq_reserve")

    def release(self, seq: int, stream=None):
        _check(lib().laser_kv_seq_release(self._h, seq, _stream(stream)), "laser_kv_seq_release")

    def import_layer(self, seq: int, layer: int, k: torch.Tensor, v: torch.Tensor, stream=None):
        n = k.shape[0]
        _check(lib().laser_kv_import(self._h, seq, layer, _dev(k, torch.float16, "k"), _dev(v, torch.float16, "v"),
                                     n, _stream(stream)), "laser_kv_import")

    def set_len(self, seq: int, n: int, stream=None):
        _check(lib().laser_kv_seq_set_len(self._h, seq, n, _stream(stream)), "laser_kv_seq_set_len")

    def read_lens(self, seq_ids, stream=None) -> np.ndarray:
        ids = _host_i32(seq_ids, "seq_ids")
        out = np.empty(ids.size, dtype=np.int32)
        _check(lib().laser_kv_read_lens(self._h, ids.ctypes.data, ids.size, out.ctypes.data, _stream(stream)),
               "laser_kv_read_lens")
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().laser_kv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        # at interpreter shutdown the HIP runtime may already be gone; the process frees everything
        if not sys.is_finalizing():
            self.close()


def verify_step(model: Model, kv: KVCache, seq_ids, pending: torch.Tensor, drafts: torch.Tensor,
                draft_len: torch.Tensor, topk: int, p: float, mode: int = MODE_RV, want_logits: bool = False,
                out=None, stream=None):
    """laser_verify_step. Returns (accept_len [B], out_tokens [B][K+1], logits [B][K+1][V] or None)."""
    ids = _host_i32(seq_ids, "seq_ids")
    B, K = drafts.shape
    dev = pending.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, K + 1), dtype=torch.int32, device=dev))
    acc, toks = out
    logits = torch.empty((B, K + 1, model.vocab), dtype=torch.float32, device=dev) if want_logits else None
    _check(lib().laser_verify_step(model._h, kv._h, ids.ctypes.data, _dev(pending, torch.int32, "pending"),
                                   _dev(drafts, torch.int32, "drafts") if K > 0 else None,
                                   _dev(draft_len, torch.int32, "draft_len"), B, K, topk, p, mode,
                                   _dev(acc, torch.int32, "accept_len"), _dev(toks, torch.int32, "out_tokens"),
                                   logits.data_ptr() if want_logits else None, _stream(stream)),
           "laser_verify_step")
    return acc, toks, logits


def verify_head(model: Model, h: torch.Tensor, drafts: torch.Tensor, draft_len: torch.Tensor, topk: int,
                p: float, mode: int = MODE_RV, want_logits: bool = False, out=None, stream=None):
    """laser_verify_head on final-normed hidden states h fp16 [B][K+1][d]."""
    B, K = drafts.shape
    if h.shape != (B, K + 1, model.d):
        raise LaserError("h must be [B][K+1][d]")
    dev = h.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, K + 1), dtype=torch.int32, device=dev))
    acc, toks = out
    logits = torch.empty((B, K + 1, model.vocab), dtype=torch.float32, device=dev) if want_logits else None
    _check(lib().laser_verify_head(model._h, _dev(h, torch.float16, "h"),
                                   _dev(drafts, torch.int32, "drafts") if K > 0 else None,
                                   _dev(draft_len, torch.int32, "draft_len"), B, K, topk, p, mode,
                                   _dev(acc, torch.int32, "accept_len"), _dev(toks, torch.int32, "out_tokens"),
                                   logits.data_ptr() if want_logits else None, _stream(stream)),
           "laser_verify_head")
    return acc, toks, logits


def retrieve_tree(pool: "Pool", keys: torch.Tensor, ctx_tail: torch.Tensor, n_min: int, n_max: int, K: int,
                  min_tokens: int = 1, out=None, stream=None):
    """laser_retrieve_tree. Returns (tree_tokens [B][K], tree_parent [B][K], tree_freq [B][K], tree_len [B], match_n [B])."""
    B = keys.shape[0]
    dev = keys.device
    if out is None:
        out = (torch.empty((B, K), dtype=torch.int32, device=dev), torch.empty((B, K), dtype=torch.int32, device=dev),
               torch.empty((B, K), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev))
    tok, par, freq, tl, mn = out
    _check(lib().laser_retrieve_tree(pool._h, _dev(keys, torch.int64, "keys"), _dev(ctx_tail, torch.int32, "ctx_tail"),
                                     B, n_min, n_max, K, min_tokens,
                                     _dev(tok, torch.int32, "tree_tokens") if K > 0 else None,
                                     _dev(par, torch.int32, "tree_parent") if K > 0 else None,
                                     (_dev(freq, torch.int32, "tree_freq") if K > 0 else None) if freq is not None else None,
                                     _dev(tl, torch.int32, "tree_len"), _dev(mn, torch.int32, "match_n"), _stream(stream)),
           "laser_retrieve_tree")
    return tok, par, freq, tl, mn


def verify_tree(model: "Model", kv: "KVCache", seq_ids, pending: torch.Tensor, tree_tokens: torch.Tensor,
                tree_parent: torch.Tensor, tree_len: torch.Tensor, topk: int, p: float, mode: int = MODE_RV,
                want_logits: bool = False, out=None, stream=None):
    """laser_verify_tree. Returns (accept_len [B], out_tokens [B][K+1], accept_path [B][K], logits or None)."""
    ids = _host_i32(seq_ids, "seq_ids")
    B, K = tree_tokens.shape
    dev = pending.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, K + 1), dtype=torch.int32, device=dev),
               torch.empty((B, K), dtype=torch.int32, device=dev))
    acc, toks, path = out
    logits = torch.empty((B, K + 1, model.vocab), dtype=torch.float32, device=dev) if want_logits else None
    _check(lib().laser_verify_tree(model._h, kv._h, ids.ctypes.data, _dev(pending, torch.int32, "pending"),
                                   _dev(tree_tokens, torch.int32, "tree_tokens") if K > 0 else None,
                                   _dev(tree_parent, torch.int32, "tree_parent") if K > 0 else None,
                                   _dev(tree_len, torch.int32, "tree_len"), B, K, topk, p, mode,
                                   _dev(acc, torch.int32, "accept_len"), _dev(toks, torch.int32, "out_tokens"),
                                   _dev(path, torch.int32, "accept_path") if K > 0 else None,
                                   logits.data_ptr() if want_logits else None, _stream(stream)), "laser_verify_tree")
    return acc, toks, path, logits


def kv_commit_tree(kv: "KVCache", seq_ids, accept_len: torch.Tensor, accept_path: torch.Tensor, stream=None):
    """laser_kv_commit_tree."""
    ids = _host_i32(seq_ids, "seq_ids")
    K = accept_path.shape[1]
    _check(lib().laser_kv_commit_tree(kv._h, ids.ctypes.data, _dev(accept_len, torch.int32, "accept_len"),
                                      _dev(accept_path, torch.int32, "accept_path") if K > 0 else None, ids.size, K,
                                      _stream(stream)), "laser_kv_commit_tree")


class GenerateOpts(C.Structure):
    _fields_ = [("K", C.c_int32), ("n_min", C.c_int32), ("n_max", C.c_int32), ("min_tokens", C.c_int32), ("tree", C.c_int32),
                ("topk", C.c_int32), ("p", C.c_float), ("mode", C.c_int32), ("max_new_tokens", C.c_int32), ("eos_token", C.c_int32),
                ("check_every", C.c_int32), ("own_cap", C.c_int32)]


def generate(model: "Model", kv: "KVCache", pool, seq_ids, keys, ctx_tail: torch.Tensor, pending: torch.Tensor, K: int, n_min: int,
             topk: int, p: float, mode: int = MODE_RV, max_new_tokens: int = 64, eos_token: int = -1, tree: bool = False,
             min_tokens: int = 1, check_every: int = 8, own_tokens=None, own_len=None, time_retrieval: bool = False, stream=None):
    """laser_generate. Returns (gen_tokens int32 [B][max_new_tokens] (-1 padded), gen_len int32 [B], counters int32 [B][4],
    steps run, summed retrieval-kernel milliseconds or None)."""
    ids = _host_i32(seq_ids, "seq_ids")
    B, n_max = ctx_tail.shape
    dev = pending.device
    gen = torch.empty((B, max_new_tokens), dtype=torch.int32, device=dev)
    glen = torch.empty(B, dtype=torch.int32, device=dev)
    cnt = torch.empty((B, 4), dtype=torch.int32, device=dev)
    own_cap = own_tokens.shape[1] if own_tokens is not None else 0
    o = GenerateOpts(K, n_min, n_max, min_tokens, int(tree), topk, p, mode, max_new_tokens, eos_token, check_every, own_cap)
    steps, ms = C.c_int(0), C.c_float(0.0)
    _check(lib().laser_generate(model._h, kv._h, pool._h if pool is not None else None, ids.ctypes.data,
                                _dev(keys, torch.int64, "keys") if keys is not None else None,
                                _dev(ctx_tail, torch.int32, "ctx_tail"), _dev(pending, torch.int32, "pending"),
                                _dev(own_tokens, torch.int32, "own_tokens") if own_tokens is not None else None,
                                _dev(own_len, torch.int32, "own_len") if own_len is not None else None,
                                ids.size, C.byref(o), gen.data_ptr(), glen.data_ptr(), cnt.data_ptr(), C.byref(steps),
                                C.byref(ms) if time_retrieval else None, _stream(stream)), "laser_generate")
    return gen, glen, cnt, steps.value, (ms.value if time_retrieval else None)


def verify_head_static(model: Model, h: torch.Tensor, drafts: torch.Tensor, draft_len: torch.Tensor, topk: int,
                       p: float, mode: int, out, stream=None):
    """laser_verify_head_static: laser_verify_head without any allocation (at most 16 rows); out = (accept_len
    int32 [B], out_tokens int32 [B][K+1]) must be given."""
    B, K = drafts.shape
    if h.shape != (B, K + 1, model.d):
        raise LaserError("h must be [B][K+1][d]")
    acc, toks = out
    _check(lib().laser_verify_head_static(model._h, _dev(h, torch.float16, "h"),
                                          _dev(drafts, torch.int32, "drafts") if K > 0 else None,
                                          _dev(draft_len, torch.int32, "draft_len"), B, K, topk, p, mode,
                                          _dev(acc, torch.int32, "accept_len"), _dev(toks, torch.int32, "out_tokens"),
                                          _stream(stream)), "laser_verify_head_static")
    return acc, toks


def kv_commit(kv: KVCache, seq_ids, accept_len: torch.Tensor, stream=None):
    """laser_kv_commit."""
    ids = _host_i32(seq_ids, "seq_ids")
    _check(lib().laser_kv_commit(kv._h, ids.ctypes.data, _dev(accept_len, torch.int32, "accept_len"), ids.size,
                                 _stream(stream)), "laser_kv_commit")


def ctx_advance(ctx_tail: torch.Tensor, pending: torch.Tensor, out_tokens: torch.Tensor, accept_len: torch.Tensor,
                stream=None):
    """laser_ctx_advance."""
    B, n_max = ctx_tail.shape
    K = out_tokens.shape[1] - 1
    _check(lib().laser_ctx_advance(_dev(ctx_tail, torch.int32, "ctx_tail"), _dev(pending, torch.int32, "pending"),
                                   _dev(out_tokens, torch.int32, "out_tokens"), _dev(accept_len, torch.int32, "accept_len"),
                                   B, K, n_max, _stream(stream)), "laser_ctx_advance")


def probe_hbm(buf: torch.Tensor, reps: int = 10, stream=None):
    """laser_probe_hbm on a caller-owned CUDA scratch tensor: (read GB/s, copy GB/s)."""
    if not (isinstance(buf, torch.Tensor) and buf.is_cuda and buf.is_contiguous()):
        raise LaserError("buf must be a contiguous CUDA tensor")
    nbytes = buf.numel() * buf.element_size()
    r, c = C.c_float(), C.c_float()
    _check(lib().laser_probe_hbm(buf.data_ptr(), nbytes - nbytes % 32, reps, _stream(stream), C.byref(r), C.byref(c)),
           "laser_probe_hbm")
    return r.value, c.value


def probe_mfma_f16(scratch: torch.Tensor, reps: int = 10, stream=None) -> float:
    """laser_probe_mfma_f16: executed TFLOP/s of a register-resident fp16 matrix-instruction loop."""
    if not (isinstance(scratch, torch.Tensor) and scratch.is_cuda and scratch.numel() * scratch.element_size() >= 4):
        raise LaserError("scratch must be a CUDA tensor of at least 4 bytes")
    t = C.c_float()
    _check(lib().laser_probe_mfma_f16(scratch.data_ptr(), reps, _stream(stream), C.byref(t)), "laser_probe_mfma_f16")
    return t.value


def probe_launch(blocks: int, reps: int = 200, stream=None) -> float:
    """laser_probe_launch: microseconds per launch of an empty kernel of `blocks` wavefronts."""
    t = C.c_float()
    _check(lib().laser_probe_launch(blocks, reps, _stream(stream), C.byref(t)), "laser_probe_launch")
    return t.value


def probe_exchange(scratch: torch.Tensor, iters: int = 200, stream=None):
    """laser_probe_exchange: (microseconds per all-to-all exchange of a cooperative launch, error count)."""
    if not (isinstance(scratch, torch.Tensor) and scratch.is_cuda and scratch.is_contiguous()):
        raise LaserError("scratch must be a contiguous CUDA tensor")
    t, e = C.c_float(), C.c_int()
    _check(lib().laser_probe_exchange(scratch.data_ptr(), scratch.numel() * scratch.element_size(), iters, _stream(stream),
                                      C.byref(t), C.byref(e)), "laser_probe_exchange")
    return t.value, e.value
