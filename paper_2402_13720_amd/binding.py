"""Thin ctypes binding of libouro.so (the C ABI declared in include/ouro.h).

Argument marshalling only: every step of the verification path runs in the HIP
kernels of the library.  PyTorch provides device memory and the stream.  There is
no fallback: if the library cannot be loaded, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libouro.so")

OURO_F32, OURO_BF16 = 0, 1
OURO_KV_ROW_MAJOR, OURO_KV_HEAD_MAJOR = 0, 1


class ouro_attn_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32),
        ("B", C.c_int32), ("T", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("max_seqlen", C.c_int32),
        ("q", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("cu_seqlens", C.c_void_p),
        ("k_blk", C.c_void_p), ("v_blk", C.c_void_p), ("meta", C.c_void_p),
        ("softmax_scale", C.c_float),
        ("out", C.c_void_p), ("lse", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("ev_start", C.c_void_p), ("ev_stop", C.c_void_p),
        ("seq_len", C.c_void_p),
        ("kv_layout", C.c_int32), ("plan_override", C.c_int32), ("cache_rows", C.c_int64),
    ]


class ouro_lmhead_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32),
        ("R", C.c_int32), ("Hd", C.c_int32), ("V", C.c_int32), ("w_layout", C.c_int32),
        ("hidden", C.c_void_p), ("w", C.c_void_p), ("argmax_out", C.c_void_p), ("max_out", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("ev_start", C.c_void_p), ("ev_stop", C.c_void_p),
    ]


class ouro_accept_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("T", C.c_int32), ("gamma", C.c_int32), ("K", C.c_int32), ("beta", C.c_int32),
        ("draft_tok", C.c_void_p), ("argmax", C.c_void_p), ("meta", C.c_void_p), ("root_pred", C.c_void_p),
        ("n_accept", C.c_void_p), ("path", C.c_void_p), ("bonus", C.c_void_p), ("accept_idx", C.c_void_p),
        ("main_A", C.c_void_p), ("phrase_A", C.c_void_p), ("n_match", C.c_void_p),
        ("match_out", C.c_void_p), ("n_seg", C.c_void_p), ("seg_start", C.c_void_p), ("seg_len", C.c_void_p),
        ("repaired", C.c_void_p),
    ]


class ouro_kv_commit_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32),
        ("B", C.c_int32), ("T", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("max_accept", C.c_int32),
        ("k_blk", C.c_void_p), ("v_blk", C.c_void_p), ("accept_idx", C.c_void_p), ("n_accept", C.c_void_p),
        ("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("cu_seqlens", C.c_void_p),
        ("seq_len", C.c_void_p), ("overflow", C.c_void_p),
        ("kv_layout", C.c_int32), ("reserved0", C.c_int32), ("cache_rows", C.c_int64),
    ]


class ouro_rope_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32),
        ("B", C.c_int32), ("T", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("base", C.c_float),
        ("q", C.c_void_p), ("k_blk", C.c_void_p), ("meta", C.c_void_p), ("cu_seqlens", C.c_void_p),
        ("seq_len", C.c_void_p), ("positions", C.c_void_p), ("qkv", C.c_void_p), ("v_blk", C.c_void_p),
    ]


class ouro_rmsnorm_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32), ("R", C.c_int32), ("Hd", C.c_int32), ("eps", C.c_float),
        ("x", C.c_void_p), ("gain", C.c_void_p), ("out", C.c_void_p),
    ]


class ouro_linear_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32), ("R", C.c_int32), ("K", C.c_int32), ("N", C.c_int32),
        ("w_layout", C.c_int32), ("epilogue", C.c_int32), ("rms_eps", C.c_float),
        ("ksplit_override", C.c_int32), ("reserved0", C.c_int32),
        ("x", C.c_void_p), ("w", C.c_void_p), ("residual", C.c_void_p), ("out", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class ouro_silu_mul_desc(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32), ("R", C.c_int32), ("F", C.c_int32),
        ("gate_up", C.c_void_p), ("out", C.c_void_p),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libouro.so is not built (%s).  Run `python -m paper_2402_13720_amd.build` "
            "(or __graft_entry__.build()) first; there is no fallback path." % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    lib.ouro_verify_attn_workspace.restype = C.c_size_t
    lib.ouro_verify_attn_workspace.argtypes = [C.POINTER(ouro_attn_desc)]
    lib.ouro_verify_attn.restype = C.c_int
    lib.ouro_verify_attn.argtypes = [C.POINTER(ouro_attn_desc), C.c_void_p]
    lib.ouro_verify_attn_plan.restype = C.c_int
    lib.ouro_verify_attn_plan.argtypes = [C.POINTER(ouro_attn_desc), C.POINTER(C.c_int32)]
    lib.ouro_lmhead_argmax_workspace.restype = C.c_size_t
    lib.ouro_lmhead_argmax_workspace.argtypes = [C.POINTER(ouro_lmhead_desc)]
    lib.ouro_lmhead_argmax.restype = C.c_int
    lib.ouro_lmhead_argmax.argtypes = [C.POINTER(ouro_lmhead_desc), C.c_void_p]
    lib.ouro_lmhead_argmax_static.restype = C.c_int
    lib.ouro_lmhead_argmax_static.argtypes = [C.POINTER(ouro_lmhead_desc), C.c_void_p]
    lib.ouro_lmhead_packed_w_bytes.restype = C.c_size_t
    lib.ouro_lmhead_packed_w_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.ouro_lmhead_pack_w.restype = C.c_int
    lib.ouro_lmhead_pack_w.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.ouro_accept.restype = C.c_int
    lib.ouro_accept.argtypes = [C.POINTER(ouro_accept_desc), C.c_void_p]
    lib.ouro_kv_commit.restype = C.c_int
    lib.ouro_kv_commit.argtypes = [C.POINTER(ouro_kv_commit_desc), C.c_void_p]
    for name, desc in (("ouro_rope_block", ouro_rope_desc), ("ouro_rmsnorm", ouro_rmsnorm_desc),
                       ("ouro_linear", ouro_linear_desc), ("ouro_silu_mul", ouro_silu_mul_desc)):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [C.POINTER(desc), C.c_void_p]
    for name in ("ouro_fold_rmsnorm_gain", "ouro_interleave_gate_up"):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.ouro_linear_workspace.restype = C.c_size_t
    lib.ouro_linear_workspace.argtypes = [C.POINTER(ouro_linear_desc)]
    lib.ouro_probe_stream_read.restype = C.c_int
    lib.ouro_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.ouro_probe_mfma_bf16.restype = C.c_int
    lib.ouro_probe_mfma_bf16.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.ouro_validate_meta_host.restype = C.c_int
    lib.ouro_validate_meta_host.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.ouro_status_string.restype = C.c_char_p
    lib.ouro_status_string.argtypes = [C.c_int]
    lib.ouro_last_hip_error.restype = C.c_int
    lib.ouro_version.restype = C.c_int
    return lib


lib = _load()


class OuroError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.ouro_status_string(status).decode()
        if status == -6:
            msg += " (hipError %d)" % lib.ouro_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, status))


def _check(status: int, where: str) -> None:
    if status != 0:
        raise OuroError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return OURO_F32
    if t.dtype == torch.bfloat16:
        return OURO_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _stream(stream) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def pack_meta(pid, boff) -> torch.Tensor:
    """(phrase_id, branch_off) int16 arrays/tensors [B,T] -> one int16 tensor [B,T,2] (the ouro_tok_meta layout)."""
    pid = torch.as_tensor(pid, dtype=torch.int16)
    boff = torch.as_tensor(boff, dtype=torch.int16)
    return torch.stack([pid, boff], dim=-1).contiguous()


def alloc_workspace(nbytes: int, device) -> torch.Tensor:
    """Scratch for partial results; contents never matter."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def plan_override(row_blocks: int = 0, chunk_keys: int = 0, four_waves: bool = False) -> int:
    """The descriptor field that forces the bf16 attention's launch shape in tests and tuning runs: row blocks per
    workgroup (1, 2, 4; 0 = the library's choice), keys per workgroup (a multiple of 128; 0 = the library's choice),
    and, for 4 row blocks, the four-wave kernel instead of the eight-wave one."""
    assert row_blocks in (0, 1, 2, 4) and chunk_keys % 128 == 0
    return row_blocks | (0x80 if four_waves else 0) | ((chunk_keys // 128) << 8)


def make_attn_desc(q, k_cache, v_cache, cu_seqlens, k_blk, v_blk, meta, out, max_seqlen,
                   lse=None, workspace=None, softmax_scale: float = 0.0, seq_len=None,
                   head_major: bool = False, plan: int = 0) -> ouro_attn_desc:
    """head_major: k_cache / v_cache are [Hkv, cache_rows, D] tensors instead of [rows, Hkv, D].
    plan: a plan_override() value (0: the library's heuristic)."""
    B, T, Hq, D = q.shape
    d = ouro_attn_desc()
    d.struct_size = C.sizeof(ouro_attn_desc)
    d.dtype = _dtype_code(q)
    d.B, d.T, d.Hq, d.Hkv, d.D = B, T, Hq, k_blk.shape[2], D
    d.max_seqlen = int(max_seqlen)
    d.q, d.k_cache, d.v_cache = _ptr(q), _ptr(k_cache), _ptr(v_cache)
    d.cu_seqlens, d.k_blk, d.v_blk, d.meta = _ptr(cu_seqlens), _ptr(k_blk), _ptr(v_blk), _ptr(meta)
    d.softmax_scale = float(softmax_scale)
    d.out, d.lse = _ptr(out), _ptr(lse)
    d.workspace = _ptr(workspace)
    d.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    d.seq_len = _ptr(seq_len)
    d.plan_override = int(plan)
    if head_major:
        d.kv_layout = OURO_KV_HEAD_MAJOR
        d.cache_rows = 0 if k_cache is None else k_cache.shape[1]
    return d


def ouro_verify_attn_workspace(q, k_blk, max_seqlen: int, plan: int = 0) -> int:
    """Workspace bytes for a call with these shapes (host-only query)."""
    B, T, Hq, D = q.shape
    d = ouro_attn_desc()
    d.struct_size = C.sizeof(ouro_attn_desc)
    d.dtype = _dtype_code(q)
    d.B, d.T, d.Hq, d.Hkv, d.D, d.max_seqlen = B, T, Hq, k_blk.shape[2], D, int(max_seqlen)
    d.plan_override = int(plan)
    return int(lib.ouro_verify_attn_workspace(C.byref(d)))


def ouro_verify_attn_plan(q, k_blk, max_seqlen: int, plan: int = 0) -> dict:
    """The launch shape a call with these shapes will use (host-only query)."""
    B, T, Hq, D = q.shape
    d = ouro_attn_desc()
    d.struct_size = C.sizeof(ouro_attn_desc)
    d.dtype = _dtype_code(q)
    d.B, d.T, d.Hq, d.Hkv, d.D, d.max_seqlen = B, T, Hq, k_blk.shape[2], D, int(max_seqlen)
    d.plan_override = int(plan)
    out = (C.c_int32 * 5)()
    _check(lib.ouro_verify_attn_plan(C.byref(d), out), "ouro_verify_attn_plan")
    return {"row_blocks_per_workgroup": out[0], "keys_per_workgroup": out[1], "chunks_per_sequence": out[2],
            "workgroups": out[3], "waves_per_workgroup": out[4]}


def ouro_verify_attn(q, k_cache, v_cache, cu_seqlens, k_blk, v_blk, meta, max_seqlen: int,
                     out=None, lse=None, workspace=None, softmax_scale: float = 0.0, stream=None, seq_len=None,
                     head_major: bool = False, plan: int = 0):
    """Masked draft-block attention.  Tensors are device tensors laid out as in include/ouro.h.
    Allocates out/workspace with torch when not given; returns out."""
    assert seq_len is None or (seq_len.dtype == torch.int32 and seq_len.is_contiguous())
    for t in (q, k_blk, v_blk):
        assert t.is_contiguous()
    assert cu_seqlens.dtype == torch.int64 and meta.dtype == torch.int16 and meta.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = ouro_verify_attn_workspace(q, k_blk, max_seqlen, plan)
        if need:
            workspace = alloc_workspace(need, q.device)
    d = make_attn_desc(q, k_cache, v_cache, cu_seqlens, k_blk, v_blk, meta, out, max_seqlen, lse, workspace,
                       softmax_scale, seq_len, head_major, plan)
    _check(lib.ouro_verify_attn(C.byref(d), _stream(stream)), "ouro_verify_attn")
    return out


OURO_W_ROW_MAJOR, OURO_W_TILED = 0, 1


class TiledWeight:
    """A bf16 LM-head weight re-blocked by ouro_lmhead_pack_w (contiguous 128 x 64 tiles)."""

    def __init__(self, data: torch.Tensor, V: int, Hd: int):
        self.data, self.V, self.Hd = data, V, Hd
        self.shape = (V, Hd)
        self.dtype = torch.bfloat16

    def data_ptr(self):
        return self.data.data_ptr()

    def is_contiguous(self):
        return True


def ouro_lmhead_pack_w(w: torch.Tensor, stream=None) -> TiledWeight:
    """Re-block a row-major bf16 weight [V, Hd] once, at load time, into the tiled layout."""
    assert w.dtype == torch.bfloat16 and w.is_contiguous()
    V, Hd = w.shape
    nbytes = int(lib.ouro_lmhead_packed_w_bytes(V, Hd))
    if nbytes == 0:
        raise OuroError(-2, "ouro_lmhead_packed_w_bytes")
    out = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=w.device)
    _check(lib.ouro_lmhead_pack_w(_ptr(w), _ptr(out), V, Hd, _stream(stream)), "ouro_lmhead_pack_w")
    return TiledWeight(out, V, Hd)


def make_lmhead_desc(hidden, w, argmax_out, max_out=None, workspace=None) -> ouro_lmhead_desc:
    d = ouro_lmhead_desc()
    d.struct_size = C.sizeof(ouro_lmhead_desc)
    d.dtype = _dtype_code(hidden)
    d.w_layout = OURO_W_TILED if isinstance(w, TiledWeight) else OURO_W_ROW_MAJOR
    d.R, d.Hd, d.V = hidden.shape[0], hidden.shape[1], w.shape[0]
    d.hidden, d.w, d.argmax_out, d.max_out = _ptr(hidden), _ptr(w), _ptr(argmax_out), _ptr(max_out)
    d.workspace = _ptr(workspace)
    d.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return d


def ouro_lmhead_argmax_workspace(hidden, w) -> int:
    d = make_lmhead_desc(hidden, w, None)
    return int(lib.ouro_lmhead_argmax_workspace(C.byref(d)))


def ouro_lmhead_argmax(hidden, w, argmax_out=None, max_out=None, workspace=None, stream=None):
    """LM head + vocabulary arg-max.  hidden [R,Hd], w [V,Hd]; returns int32 [R]."""
    assert hidden.is_contiguous() and w.is_contiguous() and hidden.dtype == w.dtype
    assert hidden.shape[1] == w.shape[1]
    if argmax_out is None:
        argmax_out = torch.empty(hidden.shape[0], dtype=torch.int32, device=hidden.device)
    if workspace is None:
        workspace = alloc_workspace(ouro_lmhead_argmax_workspace(hidden, w), hidden.device)
    d = make_lmhead_desc(hidden, w, argmax_out, max_out, workspace)
    _check(lib.ouro_lmhead_argmax(C.byref(d), _stream(stream)), "ouro_lmhead_argmax")
    return argmax_out


def ouro_lmhead_argmax_static(hidden, w, argmax_out, max_out=None, stream=None):
    """ouro_lmhead_argmax with the partials in the library's built-in buffer: no workspace, nothing allocated by the
    call (the outputs are the caller's).  Returns argmax_out."""
    assert hidden.is_contiguous() and w.is_contiguous() and hidden.dtype == w.dtype
    d = make_lmhead_desc(hidden, w, argmax_out, max_out, None)
    _check(lib.ouro_lmhead_argmax_static(C.byref(d), _stream(stream)), "ouro_lmhead_argmax_static")
    return argmax_out


def make_accept_desc(draft_tok, argmax, meta, root_pred, gamma, K, beta, outs) -> ouro_accept_desc:
    B, T = draft_tok.shape
    d = ouro_accept_desc()
    d.struct_size = C.sizeof(ouro_accept_desc)
    d.B, d.T, d.gamma, d.K, d.beta = B, T, gamma, K, beta
    d.draft_tok, d.argmax, d.meta, d.root_pred = _ptr(draft_tok), _ptr(argmax), _ptr(meta), _ptr(root_pred)
    d.n_accept, d.path, d.bonus = _ptr(outs["n_accept"]), _ptr(outs["path"]), _ptr(outs["bonus"])
    d.accept_idx = _ptr(outs["accept_idx"])
    d.main_A, d.phrase_A, d.n_match = _ptr(outs.get("main_A")), _ptr(outs.get("phrase_A")), _ptr(outs.get("n_match"))
    d.match_out, d.repaired = _ptr(outs.get("match")), _ptr(outs.get("repaired"))
    d.n_seg, d.seg_start, d.seg_len = _ptr(outs.get("n_seg")), _ptr(outs.get("seg_start")), _ptr(outs.get("seg_len"))
    return d


def alloc_pool_outputs(B: int, gamma: int, K: int, beta: int, device) -> dict:
    """Optional outputs of ouro_accept for the phrase pool; merge into the dict passed as ``outs``."""
    i32 = dict(dtype=torch.int32, device=device)
    nmax = max(1, (gamma + 1) // 2)
    return {
        "match": torch.empty(B, gamma + K * beta, dtype=torch.uint8, device=device),
        "n_seg": torch.empty(B, **i32), "seg_start": torch.empty(B, nmax, **i32), "seg_len": torch.empty(B, nmax, **i32),
        "repaired": torch.empty(B, K, beta + 1, **i32),
    }


def alloc_accept_outputs(B: int, gamma: int, K: int, beta: int, device) -> dict:
    i32 = dict(dtype=torch.int32, device=device)
    return {
        "n_accept": torch.empty(B, **i32), "path": torch.empty(B, **i32), "bonus": torch.empty(B, **i32),
        "accept_idx": torch.empty(B, gamma + beta, **i32), "main_A": torch.empty(B, **i32),
        "phrase_A": torch.empty(B, max(K, 1), **i32)[:, :K].contiguous() if K else torch.empty(B, 0, **i32),
        "n_match": torch.empty(B, **i32),
    }


def ouro_accept(draft_tok, argmax, meta, root_pred, gamma: int, K: int, beta: int, outs=None, stream=None) -> dict:
    """Longest-accepted-prefix decision.  draft_tok/argmax int32 [B,T]; returns dict of int32 tensors."""
    assert draft_tok.dtype == torch.int32 and argmax.dtype == torch.int32
    assert draft_tok.is_contiguous() and argmax.is_contiguous()
    B, T = draft_tok.shape
    if outs is None:
        outs = alloc_accept_outputs(B, gamma, K, beta, draft_tok.device)
    d = make_accept_desc(draft_tok, argmax.view(B, T), meta, root_pred, gamma, K, beta, outs)
    _check(lib.ouro_accept(C.byref(d), _stream(stream)), "ouro_accept")
    return outs


def make_kv_commit_desc(k_blk, v_blk, accept_idx, n_accept, k_cache, v_cache, cu_seqlens, seq_len,
                        overflow, head_major: bool = False) -> ouro_kv_commit_desc:
    B, T, Hkv, D = k_blk.shape
    d = ouro_kv_commit_desc()
    d.struct_size = C.sizeof(ouro_kv_commit_desc)
    d.dtype = _dtype_code(k_blk)
    d.B, d.T, d.Hkv, d.D, d.max_accept = B, T, Hkv, D, accept_idx.shape[1]
    d.k_blk, d.v_blk, d.accept_idx, d.n_accept = _ptr(k_blk), _ptr(v_blk), _ptr(accept_idx), _ptr(n_accept)
    d.k_cache, d.v_cache, d.cu_seqlens = _ptr(k_cache), _ptr(v_cache), _ptr(cu_seqlens)
    d.seq_len, d.overflow = _ptr(seq_len), _ptr(overflow)
    if head_major:
        d.kv_layout = OURO_KV_HEAD_MAJOR
        d.cache_rows = k_cache.shape[1]
    return d


def ouro_kv_commit(k_blk, v_blk, accept_idx, n_accept, k_cache, v_cache, cu_seqlens, seq_len, overflow=None,
                   stream=None, head_major: bool = False):
    """Keep the accepted block tokens: their K/V rows go to the tail of each sequence's cached tokens and
    seq_len (int32 [B]) grows in place.  Returns overflow (int32 [B])."""
    assert k_blk.is_contiguous() and v_blk.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous()
    assert accept_idx.dtype == torch.int32 and accept_idx.is_contiguous() and n_accept.dtype == torch.int32
    assert seq_len.dtype == torch.int32 and cu_seqlens.dtype == torch.int64
    assert k_cache.dtype == k_blk.dtype and v_cache.dtype == v_blk.dtype
    if overflow is None:
        overflow = torch.empty(k_blk.shape[0], dtype=torch.int32, device=k_blk.device)
    d = make_kv_commit_desc(k_blk, v_blk, accept_idx, n_accept, k_cache, v_cache, cu_seqlens, seq_len, overflow,
                            head_major)
    _check(lib.ouro_kv_commit(C.byref(d), _stream(stream)), "ouro_kv_commit")
    return overflow


def ouro_rope_block(q, k_blk, meta, cu_seqlens, seq_len=None, base: float = 0.0, positions=None, stream=None,
                    qkv=None, v_blk=None):
    """Rotary embedding of the block's q [B,T,Hq,D] and k_blk [B,T,Hkv,D] at the positions the draft structure gives
    (cached tokens + tokens before it in the token's own draft): in place, or, with qkv [B*T, (Hq+2*Hkv)*D] (a fused
    projection's output), read from there, with the value heads copied to v_blk.  Returns positions if given."""
    assert q.is_contiguous() and k_blk.is_contiguous() and q.dtype == k_blk.dtype
    if qkv is not None:
        assert v_blk is not None and v_blk.is_contiguous() and qkv.is_contiguous() and qkv.dtype == q.dtype
        assert qkv.numel() == q.numel() + k_blk.numel() + v_blk.numel() and v_blk.shape == k_blk.shape
    B, T, Hq, D = q.shape
    d = ouro_rope_desc()
    d.struct_size = C.sizeof(ouro_rope_desc)
    d.dtype = _dtype_code(q)
    d.B, d.T, d.Hq, d.Hkv, d.D = B, T, Hq, k_blk.shape[2], D
    d.base = float(base)
    d.q, d.k_blk, d.meta, d.cu_seqlens = _ptr(q), _ptr(k_blk), _ptr(meta), _ptr(cu_seqlens)
    d.seq_len, d.positions = _ptr(seq_len), _ptr(positions)
    d.qkv, d.v_blk = _ptr(qkv), _ptr(v_blk)
    _check(lib.ouro_rope_block(C.byref(d), _stream(stream)), "ouro_rope_block")
    return positions


def ouro_rmsnorm(x, gain, eps: float, out=None, stream=None):
    assert x.is_contiguous() and gain.is_contiguous() and gain.dtype == x.dtype
    if out is None:
        out = torch.empty_like(x)
    d = ouro_rmsnorm_desc()
    d.struct_size = C.sizeof(ouro_rmsnorm_desc)
    d.dtype = _dtype_code(x)
    d.R, d.Hd, d.eps = x.shape[0], x.shape[1], float(eps)
    d.x, d.gain, d.out = _ptr(x), _ptr(gain), _ptr(out)
    _check(lib.ouro_rmsnorm(C.byref(d), _stream(stream)), "ouro_rmsnorm")
    return out


OURO_EPI_NONE, OURO_EPI_SWIGLU_PAIRS = 0, 1


def ouro_interleave_gate_up(w_gate: torch.Tensor, w_up: torch.Tensor, stream=None) -> torch.Tensor:
    """[F, K] gate and up weights -> [2F, K] with rows (gate_0, up_0, gate_1, up_1, ..): the layout the
    swiglu epilogue of ouro_linear expects.  A load-time step (one library launch)."""
    assert w_gate.shape == w_up.shape and w_gate.dtype == w_up.dtype == torch.bfloat16
    assert w_gate.is_contiguous() and w_up.is_contiguous()
    F, K = w_gate.shape
    out = torch.empty(2 * F, K, dtype=w_gate.dtype, device=w_gate.device)
    _check(lib.ouro_interleave_gate_up(_ptr(w_gate), _ptr(w_up), _ptr(out), F, K, _stream(stream)),
           "ouro_interleave_gate_up")
    return out


def ouro_fold_rmsnorm_gain(w: torch.Tensor, gain: torch.Tensor, stream=None) -> torch.Tensor:
    """bf16(w[n, k] * gain[k]): the weight ouro_linear(rms_eps=...) expects.  A load-time step (one library launch)."""
    assert w.dtype == gain.dtype == torch.bfloat16 and w.is_contiguous() and gain.is_contiguous()
    N, K = w.shape
    assert gain.shape == (K,)
    out = torch.empty_like(w)
    _check(lib.ouro_fold_rmsnorm_gain(_ptr(w), _ptr(gain), _ptr(out), N, K, _stream(stream)), "ouro_fold_rmsnorm_gain")
    return out


def ouro_linear(x, w, residual=None, out=None, stream=None, workspace=None, swiglu: bool = False, rms_eps: float = 0.0,
                ksplit: int = 0):
    """out = x . w^T (+ residual); w is a [N, K] bf16 tensor or a TiledWeight.  swiglu: w holds interleaved
    (gate, up) rows and out [R, N/2] = silu(gate) * up.  rms_eps > 0: rows of the product scaled by
    1/sqrt(mean(x^2) + rms_eps) (RMSNorm of x with the gain folded into w).  ksplit > 0 forces the number of
    workgroups the k range is split over (tests, tuning)."""
    assert x.is_contiguous() and x.dtype == torch.bfloat16
    tiled = isinstance(w, TiledWeight)
    N, K = (w.V, w.Hd) if tiled else tuple(w.shape)
    assert K == x.shape[1]
    if out is None:
        out = torch.empty(x.shape[0], N // 2 if swiglu else N, dtype=x.dtype, device=x.device)
    d = ouro_linear_desc()
    d.struct_size = C.sizeof(ouro_linear_desc)
    d.dtype = OURO_BF16
    d.R, d.K, d.N = x.shape[0], K, N
    d.w_layout = OURO_W_TILED if tiled else OURO_W_ROW_MAJOR
    d.epilogue = OURO_EPI_SWIGLU_PAIRS if swiglu else OURO_EPI_NONE
    d.rms_eps = float(rms_eps)
    d.ksplit_override = int(ksplit)
    d.x, d.w, d.residual, d.out = _ptr(x), _ptr(w.data if tiled else w), _ptr(residual), _ptr(out)
    if workspace is None:
        need = int(lib.ouro_linear_workspace(C.byref(d)))
        if need:
            workspace = alloc_workspace(need, x.device)
    d.workspace = _ptr(workspace)
    d.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.ouro_linear(C.byref(d), _stream(stream)), "ouro_linear")
    return out


def ouro_silu_mul(gate_up, out=None, stream=None):
    assert gate_up.is_contiguous() and gate_up.shape[1] % 2 == 0
    R, F = gate_up.shape[0], gate_up.shape[1] // 2
    if out is None:
        out = torch.empty(R, F, dtype=gate_up.dtype, device=gate_up.device)
    d = ouro_silu_mul_desc()
    d.struct_size = C.sizeof(ouro_silu_mul_desc)
    d.dtype = _dtype_code(gate_up)
    d.R, d.F = R, F
    d.gate_up, d.out = _ptr(gate_up), _ptr(out)
    _check(lib.ouro_silu_mul(C.byref(d), _stream(stream)), "ouro_silu_mul")
    return out
