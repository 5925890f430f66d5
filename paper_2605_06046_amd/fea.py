"""ctypes binding of libfea.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

FEA_DTYPE_F32 = 0
FEA_DTYPE_BF16 = 1
FEA_FLAG_REUSE_PLAN = 1
FEA_FLAG_PLAN_ONLY = 2
FEA_FLAG_REFRESH_PLAN = 4
_CODES = {-1: "FEA_EINVAL", -2: "FEA_ENOMEM", -3: "FEA_ERANGE", -4: "FEA_EHIP"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None


class FeaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{_CODES.get(code, code)}: {message}")
        self.code = code


class AttnParams(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float),
                ("split_blocks", C.c_int32), ("max_group", C.c_int32), ("flags", C.c_int32),
                ("run_kernel_min", C.c_int32), ("merge_rows_min", C.c_int32), ("fused_max", C.c_int32)]

    def __init__(self, num_q_heads, num_kv_heads, head_dim, dtype, scale=0.0, split_blocks=0,
                 max_group=0, flags=0, block_size=16, run_kernel_min=0, merge_rows_min=0, fused_max=0):
        super().__init__(num_q_heads, num_kv_heads, head_dim, block_size, dtype, scale,
                         split_blocks, max_group, flags, run_kernel_min, merge_rows_min, fused_max)


def library_path() -> str:
    """The in-tree build; FEA_LIBRARY names another build of the same library (development aid)."""
    return os.environ.get("FEA_LIBRARY") or os.path.join(_HERE, "libfea.so")


class StopPolicy(C.Structure):
    """fea_stop_policy: the five constants of the rule-based stop policy."""
    _fields_ = [("small_batch", C.c_int32), ("loss_small", C.c_int32), ("loss_limit", C.c_int32),
                ("peers_relax", C.c_int32), ("loss_relaxed", C.c_int32)]


FEA_ADD, FEA_STOP = 0, 1
FEA_HASH_CHAINED, FEA_HASH_XXH64 = 0, 1
FEA_POLICY_UCB, FEA_POLICY_QLEARN = 1, 2


class PolicyParams(C.Structure):
    """fea_policy_params: kind, bins and constants of a learned stop policy."""
    _fields_ = [("kind", C.c_int32), ("b_bins", C.c_int32), ("w_bins", C.c_int32),
                ("n_loss_thresholds", C.c_int32), ("loss_thresholds", C.c_int32 * 8),
                ("reward_every_step", C.c_int32), ("c", C.c_double), ("alpha", C.c_double),
                ("gamma", C.c_double), ("eps", C.c_double), ("eps_min", C.c_double), ("eps_decay", C.c_double)]


def load_library() -> C.CDLL:
    """Loads libfea.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime.  Whichever copy is mapped first serves the whole
    # process, and device work only lines up with the caller's tensors and streams if
    # it is PyTorch's: bring it in before libfea.so resolves its libamdhip64 dependency.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2605_06046_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
    sigs = {
        "fea_last_error": (C.c_char_p, []),
        "fea_kv_alloc": (i32, [u32, u32, u64, C.POINTER(vp)]),
        "fea_kv_free": (i32, [vp]),
        "fea_kv_stats": (i32, [vp, C.POINTER(u32), C.POINTER(u32), C.POINTER(u32), vp]),
        "fea_chunk_hashes": (i32, [vp, i64, vp]),
        "fea_chunk_hashes_xxh64": (i32, [vp, i64, u64, vp]),
        "fea_kv_set_hash": (i32, [vp, i32, u64]),
        "fea_chunk_hashes_device": (i32, [vp, i64, vp, i32, vp, vp, i64, vp]),
        "fea_cht_set_hash": (i32, [vp, i32, u64]),
        "fea_build_block_tables": (i32, [vp, vp, vp, i32, i32, vp, vp, vp, vp]),
        "fea_release": (i32, [vp, vp, i32]),
        "fea_validate_block_tables": (i32, [vp, i32, vp, i32, u32]),
        "fea_decode_workspace_bytes": (i32, [C.POINTER(AttnParams), i32, i32, C.POINTER(C.c_size_t)]),
        "fea_decode_attention": (i32, [C.POINTER(AttnParams), vp, vp, vp, vp, i32, vp, i32, vp, vp, C.c_size_t, vp]),
        "fea_decode_attention_static": (i32, [C.POINTER(AttnParams), vp, vp, vp, vp, i32, vp, i32, vp, vp]),
        "fea_decode_plan_info": (i32, [vp, vp, vp]),
        "fea_stream_read_gbs": (i32, [vp, C.c_size_t, i32, i32, vp, C.POINTER(C.c_double)]),
        "fea_profile_enable": (i32, [i32, i32]),
        "fea_profile_read": (i32, [i32, vp]),
        "fea_kv_extend": (i32, [vp, vp, i32, vp, i32, C.POINTER(i32)]),
        "fea_kv_append": (i32, [C.POINTER(AttnParams), vp, vp, vp, vp, vp, i32, vp, i32, vp]),
        "fea_cht_create": (i32, [i32, C.POINTER(vp)]),
        "fea_cht_destroy": (None, [vp]),
        "fea_cht_insert": (i32, [vp, i64, vp, i64]),
        "fea_cht_insert_hashes": (i32, [vp, i64, vp, i32]),
        "fea_cht_find_best": (i32, [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "fea_cht_add_to_batch": (i32, [vp, i64]),
        "fea_cht_finish": (i32, [vp, i64]),
        "fea_cht_remove": (i32, [vp, i64]),
        "fea_cht_missing": (i32, [vp, i64, C.POINTER(i32)]),
        "fea_cht_stats": (i32, [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(u64), C.POINTER(i64), C.POINTER(i64)]),
        "fea_cht_build_batch": (i32, [vp, C.POINTER(StopPolicy), i32, vp, C.POINTER(i32)]),
        "fea_policy_create": (i32, [C.POINTER(PolicyParams), C.POINTER(vp)]),
        "fea_policy_destroy": (None, [vp]),
        "fea_policy_state": (i32, [vp, i32, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "fea_policy_decide": (i32, [vp, i32, i32, i32, C.c_double, C.c_double, C.POINTER(i32)]),
        "fea_policy_reward": (i32, [vp, C.c_double]),
        "fea_policy_entry": (i32, [vp, i32, i32, i32, i32, C.POINTER(C.c_double), C.POINTER(i64)]),
        "fea_policy_info": (i32, [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(i32)]),
        "fea_cht_build_batch_learned": (i32, [vp, vp, i32, vp, vp, C.POINTER(i32)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise FeaError(rc, load_library().fea_last_error().decode())


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class KVPool:
    """Opaque handle of the host-side block pool."""

    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        try:
            fea_kv_free(self)
        except Exception:
            pass


def fea_kv_alloc(num_blocks: int, block_size: int = 16, perm_seed: int = 0) -> KVPool:
    h = C.c_void_p()
    _check(load_library().fea_kv_alloc(num_blocks, block_size, perm_seed, C.byref(h)))
    return KVPool(h)


def fea_kv_free(pool: KVPool) -> None:
    if pool.handle:
        load_library().fea_kv_free(pool.handle)
        pool.handle = None


def fea_kv_stats(pool: KVPool):
    """(num_blocks, free_blocks, hash_collisions, refcounts[int32])"""
    lib = load_library()
    nb, fb, col = C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(lib.fea_kv_stats(pool.handle, C.byref(nb), C.byref(fb), C.byref(col), None))
    rc = np.zeros(nb.value, dtype=np.int32)
    _check(lib.fea_kv_stats(pool.handle, None, None, None, _np_ptr(rc)))
    return nb.value, fb.value, col.value, rc


def fea_chunk_hashes(tokens: np.ndarray) -> np.ndarray:
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    out = np.zeros(-(-len(tokens) // 16), dtype=np.uint64)
    _check(load_library().fea_chunk_hashes(_np_ptr(tokens), len(tokens), _np_ptr(out)))
    return out


def fea_chunk_hashes_xxh64(tokens: np.ndarray, seed: int = 0) -> np.ndarray:
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    out = np.zeros(-(-len(tokens) // 16), dtype=np.uint64)
    _check(load_library().fea_chunk_hashes_xxh64(_np_ptr(tokens), len(tokens), seed, _np_ptr(out)))
    return out


def fea_kv_set_hash(pool: KVPool, kind: int, seed: int = 0) -> None:
    _check(load_library().fea_kv_set_hash(pool.handle, kind, seed))


def fea_build_block_tables(pool: KVPool, tokens: np.ndarray, tok_offsets: np.ndarray,
                           max_blocks_per_seq: int, want_hashes: bool = False):
    """Returns (block_tables[B, max_blocks] int32, seq_lens[B] int32, hashes, hash_offsets)."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    tok_offsets = np.ascontiguousarray(tok_offsets, dtype=np.int64)
    B = len(tok_offsets) - 1
    tables = np.full((B, max_blocks_per_seq), -2, dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    hashes = hoff = None
    if want_hashes:
        total = int(sum(-(-int(t) // 16) for t in np.diff(tok_offsets)))
        hashes = np.zeros(total, dtype=np.uint64)
        hoff = np.zeros(B + 1, dtype=np.int64)
    _check(load_library().fea_build_block_tables(pool.handle, _np_ptr(tokens), _np_ptr(tok_offsets), B,
                                                 max_blocks_per_seq, _np_ptr(tables), _np_ptr(lens),
                                                 _np_ptr(hashes), _np_ptr(hoff)))
    return tables, lens, hashes, hoff


def fea_release(pool: KVPool, row: np.ndarray) -> None:
    row = np.ascontiguousarray(row, dtype=np.int32)
    _check(load_library().fea_release(pool.handle, _np_ptr(row), len(row)))


def fea_kv_extend(pool: KVPool, tables: np.ndarray, seq_lens: np.ndarray) -> int:
    """One decode step of bookkeeping, in place on the C-contiguous int32 host arrays; returns the blocks added."""
    assert tables.dtype == np.int32 and seq_lens.dtype == np.int32 and tables.flags.c_contiguous and seq_lens.flags.c_contiguous
    n = C.c_int32()
    _check(load_library().fea_kv_extend(pool.handle, _np_ptr(tables), tables.shape[1], _np_ptr(seq_lens),
                                        tables.shape[0], C.byref(n)))
    return n.value


def fea_validate_block_tables(tables: np.ndarray, seq_lens: np.ndarray, num_blocks: int) -> None:
    tables = np.ascontiguousarray(tables, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    _check(load_library().fea_validate_block_tables(_np_ptr(tables), tables.shape[1], _np_ptr(seq_lens),
                                                    tables.shape[0], num_blocks))


def fea_decode_workspace_bytes(params: AttnParams, B: int, table_stride: int) -> int:
    out = C.c_size_t()
    _check(load_library().fea_decode_workspace_bytes(C.byref(params), B, table_stride, C.byref(out)))
    return out.value


def _dev_ptr(t):
    return C.c_void_p(t.data_ptr())


def fea_decode_attention(params: AttnParams, q, k_cache, v_cache, block_tables, seq_lens, out, workspace,
                         stream=None) -> None:
    """All tensor arguments are contiguous torch tensors on the GPU; `stream` is a
    torch.cuda.Stream (default: the current one).  Asynchronous."""
    import torch
    for name, t in (("q", q), ("k_cache", k_cache), ("v_cache", v_cache), ("block_tables", block_tables),
                    ("seq_lens", seq_lens), ("out", out), ("workspace", workspace)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous GPU tensor")
    if block_tables.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise ValueError("block_tables and seq_lens must be int32")
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().fea_decode_attention(
        C.byref(params), _dev_ptr(q), _dev_ptr(k_cache), _dev_ptr(v_cache), _dev_ptr(block_tables),
        block_tables.shape[1], _dev_ptr(seq_lens), q.shape[0], _dev_ptr(out), _dev_ptr(workspace),
        workspace.numel() * workspace.element_size(), C.c_void_p(st.cuda_stream)))


def fea_decode_attention_static(params: AttnParams, q, k_cache, v_cache, block_tables, seq_lens, out, stream=None) -> None:
    """fea_decode_attention on the library's built-in workspace (allocates nothing).  Asynchronous."""
    import torch
    for name, t in (("q", q), ("k_cache", k_cache), ("v_cache", v_cache), ("block_tables", block_tables),
                    ("seq_lens", seq_lens), ("out", out)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous GPU tensor")
    if block_tables.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise ValueError("block_tables and seq_lens must be int32")
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().fea_decode_attention_static(
        C.byref(params), _dev_ptr(q), _dev_ptr(k_cache), _dev_ptr(v_cache), _dev_ptr(block_tables),
        block_tables.shape[1], _dev_ptr(seq_lens), q.shape[0], _dev_ptr(out), C.c_void_p(st.cuda_stream)))


def fea_chunk_hashes_device(tokens, tok_offsets, hash_offsets, hashes, stream=None) -> None:
    """Contiguous GPU tensors: tokens int32 [n], tok_offsets and hash_offsets int64 [B+1], hashes int64 [m]
    (the 64-bit values, to be viewed as unsigned).  Asynchronous."""
    import torch
    if tokens.dtype != torch.int32 or tok_offsets.dtype != torch.int64 or hash_offsets.dtype != torch.int64 \
            or hashes.dtype != torch.int64 or tok_offsets.numel() != hash_offsets.numel():
        raise ValueError("tokens int32; tok_offsets, hash_offsets (equal lengths) and hashes int64")
    for t in (tokens, tok_offsets, hash_offsets, hashes):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("all arguments must be contiguous GPU tensors")
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().fea_chunk_hashes_device(_dev_ptr(tokens), tokens.numel(), _dev_ptr(tok_offsets),
                                                  tok_offsets.numel() - 1, _dev_ptr(hash_offsets), _dev_ptr(hashes),
                                                  hashes.numel(), C.c_void_p(st.cuda_stream)))


def fea_decode_plan_info(workspace, stream=None) -> dict:
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    info = np.zeros(9, dtype=np.int32)
    _check(load_library().fea_decode_plan_info(_dev_ptr(workspace), C.c_void_p(st.cuda_stream), _np_ptr(info)))
    keys = ("items", "groups", "grouped_requests", "split_blocks", "partial_rows", "shared_blocks",
            "variant", "overflow", "shares")
    return dict(zip(keys, (int(x) for x in info)))


def fea_kv_append(params: AttnParams, k_new, v_new, k_cache, v_cache, block_tables, seq_lens, stream=None) -> None:
    """Torch tensors on the GPU; writes each request's new K/V rows at position seq_lens - 1.  Asynchronous."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().fea_kv_append(C.byref(params), _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(k_cache),
                                        _dev_ptr(v_cache), _dev_ptr(block_tables), block_tables.shape[1],
                                        _dev_ptr(seq_lens), block_tables.shape[0], C.c_void_p(st.cuda_stream)))


def fea_stream_read_gbs(buffer, scattered: bool = True, repeats: int = 5, stream=None) -> float:
    """GB/s at which the GPU streams the contiguous GPU tensor `buffer` through the sweep's fetch path."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    out = C.c_double()
    _check(load_library().fea_stream_read_gbs(_dev_ptr(buffer), buffer.numel() * buffer.element_size(), int(bool(scattered)),
                                              int(repeats), C.c_void_p(st.cuda_stream), C.byref(out)))
    return out.value


def fea_profile_enable(max_calls: int, which: int = -1) -> None:
    """Attach timing events to the launches of the next calls (which: -1 all, 0 plan, 1 sweep, 2 merge)."""
    _check(load_library().fea_profile_enable(int(max_calls), int(which)))


def fea_profile_read(call: int):
    """(plan_ms, sweep_ms, merge_ms) of the call-th fea_decode_attention since profiling was enabled."""
    ms = np.zeros(3, dtype=np.float32)
    _check(load_library().fea_profile_read(call, _np_ptr(ms)))
    return float(ms[0]), float(ms[1]), float(ms[2])


class Cht:
    """fea_cht_*: the scheduler's Chunked Hash Tree (argument marshalling only)."""

    def __init__(self, chunk_tokens: int = 16):
        self._lib = load_library()
        h = C.c_void_p()
        _check(self._lib.fea_cht_create(chunk_tokens, C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.fea_cht_destroy(self._h)
            self._h = None

    __del__ = close

    def set_hash(self, kind: int, seed: int = 0):
        _check(self._lib.fea_cht_set_hash(self._h, kind, seed))

    def insert(self, rid: int, tokens=None, hash_vector=None):
        if hash_vector is not None:
            hv = np.ascontiguousarray(hash_vector, dtype=np.uint64)
            _check(self._lib.fea_cht_insert_hashes(self._h, rid, _np_ptr(hv), hv.size))
        else:
            tk = np.ascontiguousarray(tokens, dtype=np.int32)
            _check(self._lib.fea_cht_insert(self._h, rid, _np_ptr(tk), tk.size))

    def find_best(self):
        """(request, tip depth now, tip depth with it added, peers, missing count) or None."""
        rid, a, b, p, m = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        rc = self._lib.fea_cht_find_best(self._h, C.byref(rid), C.byref(a), C.byref(b), C.byref(p), C.byref(m))
        if rc == 1:
            return None
        _check(rc)
        return rid.value, a.value, b.value, p.value, m.value

    def add_to_batch(self, rid: int):
        _check(self._lib.fea_cht_add_to_batch(self._h, rid))

    def finish(self, rid: int):
        _check(self._lib.fea_cht_finish(self._h, rid))

    def remove(self, rid: int):
        _check(self._lib.fea_cht_remove(self._h, rid))

    def missing(self, rid: int) -> int:
        m = C.c_int32()
        _check(self._lib.fea_cht_missing(self._h, rid, C.byref(m)))
        return m.value

    def stats(self):
        nw, na, ws, he = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        tl, th = C.c_int32(), C.c_uint64()
        _check(self._lib.fea_cht_stats(self._h, C.byref(nw), C.byref(na), C.byref(tl), C.byref(th), C.byref(ws), C.byref(he)))
        return {"waiting": nw.value, "active": na.value, "tip_level": tl.value, "tip_hash": th.value,
                "working_set": ws.value, "heap_entries": he.value}

    def build_batch(self, max_batch: int, **policy):
        pol = StopPolicy(**policy)
        ids = np.zeros(max(max_batch, 1), dtype=np.int64)
        n = C.c_int32()
        _check(self._lib.fea_cht_build_batch(self._h, C.byref(pol), max_batch, _np_ptr(ids), C.byref(n)))
        return ids[:n.value].tolist()

    def build_batch_learned(self, policy: "Policy", max_batch: int, draws=None):
        """fea_cht_build_batch_learned; draws: [max_batch, 2] uniforms (None for the bandit)."""
        ids = np.zeros(max(max_batch, 1), dtype=np.int64)
        n = C.c_int32()
        d = None
        if draws is not None:
            d = np.ascontiguousarray(draws, dtype=np.float64).reshape(-1)
            if d.size < 2 * max_batch:
                raise ValueError("draws must hold 2 * max_batch values")
        _check(self._lib.fea_cht_build_batch_learned(self._h, policy._h, max_batch, _np_ptr(d), _np_ptr(ids), C.byref(n)))
        return ids[:n.value].tolist()


class Policy:
    """fea_policy_*: a learned stop policy (argument marshalling only)."""

    def __init__(self, kind: int, b_bins: int, w_bins: int, loss_thresholds=(), c: float = 0.0, alpha: float = 0.0,
                 gamma: float = 0.0, eps: float = 0.0, eps_min: float = 0.0, eps_decay: float = 1.0,
                 reward_every_step: bool = True):
        self._lib = load_library()
        self._h = None
        thr = list(loss_thresholds)
        if len(thr) > 8:
            raise ValueError("at most 8 loss thresholds")
        prm = PolicyParams(kind, b_bins, w_bins, len(thr), (C.c_int32 * 8)(*thr), int(reward_every_step),
                           c, alpha, gamma, eps, eps_min, eps_decay)
        h = C.c_void_p()
        _check(self._lib.fea_policy_create(C.byref(prm), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.fea_policy_destroy(self._h)
            self._h = None

    __del__ = close

    def state(self, b: int, loss: int, peers: int):
        sb, sl, sw = C.c_int32(), C.c_int32(), C.c_int32()
        _check(self._lib.fea_policy_state(self._h, b, loss, peers, C.byref(sb), C.byref(sl), C.byref(sw)))
        return sb.value, sl.value, sw.value

    def decide(self, b: int, loss: int, peers: int, u_explore: float = 0.0, u_action: float = 0.0) -> int:
        a = C.c_int32()
        _check(self._lib.fea_policy_decide(self._h, b, loss, peers, u_explore, u_action, C.byref(a)))
        return a.value

    def reward(self, r: float):
        _check(self._lib.fea_policy_reward(self._h, r))

    def entry(self, state, action: int):
        v, n = C.c_double(), C.c_int64()
        _check(self._lib.fea_policy_entry(self._h, state[0], state[1], state[2], action, C.byref(v), C.byref(n)))
        return v.value, n.value

    def info(self):
        d, e, eps, o = C.c_int64(), C.c_int64(), C.c_double(), C.c_int32()
        _check(self._lib.fea_policy_info(self._h, C.byref(d), C.byref(e), C.byref(eps), C.byref(o)))
        return {"decisions": d.value, "episodes": e.value, "eps": eps.value, "open": o.value}
