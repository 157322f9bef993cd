"""Thin ctypes binding of libtyphoon_mla.so (declared in include/typhoon_mla.h).

Argument marshalling only: every step of the decode path runs in the HIP kernels of the library.
PyTorch supplies device memory (tensors) and the current HIP stream; nothing here computes.
There is no fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os
from ctypes import (POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t,
                    c_void_p)

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtyphoon_mla.so")

(TMLA_OK, TMLA_ERR_INVALID_ARG, TMLA_ERR_UNSUPPORTED, TMLA_ERR_WORKSPACE_TOO_SMALL, TMLA_ERR_HIP,
 TMLA_ERR_SCRATCH_LIMIT) = range(6)
STATIC_SCRATCH_BYTES = 128 << 20
MODE_MIXED, MODE_NAIVE_ONLY, MODE_ABSORB_ONLY, MODE_AUTO = 0, 1, 2, 3
MODES = {"mixed": MODE_MIXED, "naive_only": MODE_NAIVE_ONLY, "absorb_only": MODE_ABSORB_ONLY,
         "auto": MODE_AUTO}
BF16, FP32 = 0, 1

EXPORTS = [
    "typhoon_mla_status_string", "typhoon_mla_expanded_k_bytes", "typhoon_mla_expanded_v_bytes",
    "typhoon_mla_expand_prefix", "typhoon_mla_expand_pool", "typhoon_mla_decode_workspace_bytes",
    "typhoon_mla_decode", "typhoon_mla_combine_lse", "typhoon_mla_set_debug_flags",
    "typhoon_mla_auto_batch_threshold", "typhoon_mla_decode_tree_workspace_bytes",
    "typhoon_mla_decode_tree", "typhoon_mla_set_tuning", "typhoon_mla_decode_static_scratch",
]
TUNE_PREFIX_SPLITS, TUNE_SUFFIX_CHUNK, TUNE_ABSORB_PREFIX_CHUNK, TUNE_NAIVE_SUFFIX_CHUNK = range(4)


class tmla_dims(Structure):
    _fields_ = [("num_heads", c_int32), ("kv_lora_rank", c_int32), ("qk_nope_dim", c_int32),
                ("qk_rope_dim", c_int32), ("v_head_dim", c_int32), ("sm_scale", c_float),
                ("dtype", c_int32)]


class tmla_prefix_node(Structure):
    _fields_ = [("k", c_void_p), ("v", c_void_p), ("len", c_int32), ("level", c_int32),
                ("batch_begin", c_int32), ("batch_count", c_int32)]


def make_dims(num_heads, sm_scale, dtype, kv_lora_rank=512, qk_nope_dim=128, qk_rope_dim=64,
              v_head_dim=128):
    if isinstance(dtype, torch.dtype):
        dtype = {torch.bfloat16: BF16, torch.float32: FP32}[dtype]
    elif isinstance(dtype, str):
        dtype = {"bf16": BF16, "fp32": FP32}[dtype]
    return tmla_dims(num_heads, kv_lora_rank, qk_nope_dim, qk_rope_dim, v_head_dim, sm_scale, dtype)


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                "libtyphoon_mla.so is not built (%s); run `python -c 'import __graft_entry__ as g; "
                "g.build()'` -- there is no fallback implementation" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        P = POINTER(tmla_dims)
        L.typhoon_mla_status_string.restype = c_char_p
        L.typhoon_mla_status_string.argtypes = [c_int]
        for f in (L.typhoon_mla_expanded_k_bytes, L.typhoon_mla_expanded_v_bytes):
            f.restype = c_size_t
            f.argtypes = [P, c_int64]
        L.typhoon_mla_expand_prefix.restype = c_int
        L.typhoon_mla_expand_prefix.argtypes = [P, c_int32] + [c_void_p] * 7
        L.typhoon_mla_expand_pool.restype = c_int
        L.typhoon_mla_expand_pool.argtypes = [P, c_int32, c_int32] + [c_void_p] * 6
        L.typhoon_mla_decode_workspace_bytes.restype = c_size_t
        L.typhoon_mla_decode_workspace_bytes.argtypes = [P] + [c_int32] * 5
        L.typhoon_mla_decode.restype = c_int
        L.typhoon_mla_decode.argtypes = (
            [P, c_int32, c_int32, c_int32, c_void_p, c_int32] + [c_void_p] * 4 +
            [c_void_p, c_int32, c_int32, c_void_p, c_int32, c_void_p, c_int32] +
            [c_void_p] * 4 + [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p])
        L.typhoon_mla_decode_static_scratch.restype = c_int
        L.typhoon_mla_decode_static_scratch.argtypes = (
            [P, c_int32, c_int32, c_int32, c_void_p, c_int32] + [c_void_p] * 4 +
            [c_void_p, c_int32, c_int32, c_void_p, c_int32, c_void_p, c_int32] +
            [c_void_p] * 4 + [c_void_p, c_void_p, c_void_p])
        L.typhoon_mla_combine_lse.restype = c_int
        L.typhoon_mla_combine_lse.argtypes = [c_int32, c_int64, c_int32, c_void_p, c_void_p,
                                              c_void_p, c_int32, c_void_p, c_void_p]
        L.typhoon_mla_auto_batch_threshold.restype = ctypes.c_double
        L.typhoon_mla_auto_batch_threshold.argtypes = [P, c_int32, c_int32]
        N = POINTER(tmla_prefix_node)
        L.typhoon_mla_decode_tree_workspace_bytes.restype = c_size_t
        L.typhoon_mla_decode_tree_workspace_bytes.argtypes = [P, c_int32, c_int32, N, c_int32,
                                                              c_int32]
        L.typhoon_mla_decode_tree.restype = c_int
        L.typhoon_mla_decode_tree.argtypes = (
            [P, c_int32, c_int32, c_void_p, N, c_int32, c_void_p, c_int32, c_int32, c_void_p,
             c_int32, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
             c_size_t, c_void_p])
        L.typhoon_mla_set_debug_flags.restype = c_int
        L.typhoon_mla_set_debug_flags.argtypes = [c_int]
        L.typhoon_mla_set_tuning.restype = c_int
        L.typhoon_mla_set_tuning.argtypes = [c_int, c_int]
        _lib = L
    return _lib


class TyphoonMLAError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (
            where, lib().typhoon_mla_status_string(status).decode(), status))


def _check(status, where):
    if status != TMLA_OK:
        raise TyphoonMLAError(status, where)


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors passed to the library must be dense"
    return c_void_p(t.data_ptr())


def _stream(device):
    return c_void_p(torch.cuda.current_stream(device).cuda_stream)


def typhoon_mla_status_string(status):
    return lib().typhoon_mla_status_string(int(status)).decode()


def typhoon_mla_set_debug_flags(flags):
    return lib().typhoon_mla_set_debug_flags(int(flags))


def typhoon_mla_set_tuning(key, value):
    old = lib().typhoon_mla_set_tuning(int(key), int(value))
    if old < 0:
        raise ValueError("typhoon_mla_set_tuning: unknown key %r or negative value %r" % (key, value))
    return old


def typhoon_mla_auto_batch_threshold(dims, q_len=1, prefix_len=4096):
    return lib().typhoon_mla_auto_batch_threshold(ctypes.byref(dims), int(q_len), int(prefix_len))


def typhoon_mla_expanded_k_bytes(dims, num_tokens):
    return lib().typhoon_mla_expanded_k_bytes(ctypes.byref(dims), int(num_tokens))


def typhoon_mla_expanded_v_bytes(dims, num_tokens):
    return lib().typhoon_mla_expanded_v_bytes(ctypes.byref(dims), int(num_tokens))


def _alloc_expanded(dims, ntok, device):
    kb = typhoon_mla_expanded_k_bytes(dims, ntok)
    vb = typhoon_mla_expanded_v_bytes(dims, ntok)
    k = torch.empty(max(kb, 16), dtype=torch.uint8, device=device)
    v = torch.empty(max(vb, 16), dtype=torch.uint8, device=device)
    return k, v


def typhoon_mla_expand_prefix(dims, prefix_ckv, prefix_krope, w_uk, w_uv, prefix_k=None,
                              prefix_v=None):
    """Returns (prefix_k, prefix_v): opaque byte tensors in the library's expanded layout."""
    L = prefix_ckv.shape[0]
    if prefix_k is None:
        prefix_k, prefix_v = _alloc_expanded(dims, L, prefix_ckv.device)
    st = lib().typhoon_mla_expand_prefix(ctypes.byref(dims), L, _ptr(prefix_ckv),
                                         _ptr(prefix_krope), _ptr(w_uk), _ptr(w_uv),
                                         _ptr(prefix_k), _ptr(prefix_v), _stream(w_uk.device))
    _check(st, "typhoon_mla_expand_prefix")
    return prefix_k, prefix_v


def typhoon_mla_expand_pool(dims, suffix_pool, w_uk, w_uv, suffix_k_pool=None, suffix_v_pool=None):
    nb, bs = suffix_pool.shape[0], suffix_pool.shape[1]
    if suffix_k_pool is None:
        suffix_k_pool, suffix_v_pool = _alloc_expanded(dims, nb * bs, suffix_pool.device)
    st = lib().typhoon_mla_expand_pool(ctypes.byref(dims), nb, bs, _ptr(suffix_pool), _ptr(w_uk),
                                       _ptr(w_uv), _ptr(suffix_k_pool), _ptr(suffix_v_pool),
                                       _stream(w_uk.device))
    _check(st, "typhoon_mla_expand_pool")
    return suffix_k_pool, suffix_v_pool


def typhoon_mla_decode_workspace_bytes(dims, mode, batch, q_len, prefix_len, max_suffix_len):
    return lib().typhoon_mla_decode_workspace_bytes(ctypes.byref(dims), int(mode), batch, q_len,
                                                    prefix_len, max_suffix_len)


def typhoon_mla_decode(dims, mode, q, prefix_len, prefix_k=None, prefix_v=None, prefix_ckv=None,
                       prefix_krope=None, suffix_pool=None, block_table=None, suffix_lens=None,
                       max_suffix_len=0, suffix_k_pool=None, suffix_v_pool=None, w_uk=None,
                       w_uv=None, out=None, lse_out=None, workspace=None, block_size=None,
                       num_blocks=None, want_lse=True):
    """One decode step; returns (out [B, S_q, H, 128], lse [B, S_q, H] or None)."""
    mode = MODES[mode] if isinstance(mode, str) else int(mode)
    B, S_q, H, _ = q.shape
    dev = q.device
    if out is None:
        out = torch.empty((B, S_q, H, 128), dtype=q.dtype, device=dev)
    if lse_out is None and want_lse:
        lse_out = torch.empty((B, S_q, H), dtype=torch.float32, device=dev)
    if workspace is None:
        nbytes = typhoon_mla_decode_workspace_bytes(dims, mode, B, S_q, prefix_len, max_suffix_len)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    pool_like = suffix_pool if suffix_pool is not None else None
    if num_blocks is None:
        num_blocks = pool_like.shape[0] if pool_like is not None else 0
    if block_size is None:
        block_size = pool_like.shape[1] if pool_like is not None else 64
    max_blocks = block_table.shape[1] if block_table is not None else 0
    st = lib().typhoon_mla_decode(
        ctypes.byref(dims), mode, B, S_q, _ptr(q), prefix_len, _ptr(prefix_k), _ptr(prefix_v),
        _ptr(prefix_ckv), _ptr(prefix_krope), _ptr(suffix_pool), num_blocks, block_size,
        _ptr(block_table), max_blocks, _ptr(suffix_lens), max_suffix_len, _ptr(suffix_k_pool),
        _ptr(suffix_v_pool), _ptr(w_uk), _ptr(w_uv), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel(), _stream(dev))
    _check(st, "typhoon_mla_decode")
    return out, lse_out


def typhoon_mla_decode_static_scratch(dims, mode, q, prefix_len, out, lse_out=None, prefix_k=None,
                                      prefix_v=None, prefix_ckv=None, prefix_krope=None,
                                      suffix_pool=None, block_table=None, suffix_lens=None,
                                      max_suffix_len=0, suffix_k_pool=None, suffix_v_pool=None,
                                      w_uk=None, w_uv=None):
    """typhoon_mla_decode on the library's static scratch array: nothing is allocated here or in
    the library, so `out` (and `lse_out`, if wanted) are the caller's."""
    mode = MODES[mode] if isinstance(mode, str) else int(mode)
    B, S_q, H, _ = q.shape
    num_blocks = suffix_pool.shape[0] if suffix_pool is not None else 0
    block_size = suffix_pool.shape[1] if suffix_pool is not None else 64
    max_blocks = block_table.shape[1] if block_table is not None else 0
    st = lib().typhoon_mla_decode_static_scratch(
        ctypes.byref(dims), mode, B, S_q, _ptr(q), prefix_len, _ptr(prefix_k), _ptr(prefix_v),
        _ptr(prefix_ckv), _ptr(prefix_krope), _ptr(suffix_pool), num_blocks, block_size,
        _ptr(block_table), max_blocks, _ptr(suffix_lens), max_suffix_len, _ptr(suffix_k_pool),
        _ptr(suffix_v_pool), _ptr(w_uk), _ptr(w_uv), _ptr(out), _ptr(lse_out), _stream(q.device))
    _check(st, "typhoon_mla_decode_static_scratch")
    return out, lse_out


def typhoon_mla_combine_lse(partial_out, partial_lse, out_dtype=torch.float32, want_lse=True):
    n, rows, width = partial_out.shape
    dev = partial_out.device
    out = torch.empty((rows, width), dtype=out_dtype, device=dev)
    lse = torch.empty((rows,), dtype=torch.float32, device=dev) if want_lse else None
    code = {torch.bfloat16: BF16, torch.float32: FP32}[out_dtype]
    st = lib().typhoon_mla_combine_lse(n, rows, width, _ptr(partial_out), _ptr(partial_lse),
                                       _ptr(out), code, _ptr(lse), _stream(dev))
    _check(st, "typhoon_mla_combine_lse")
    return out, lse


def make_nodes(nodes):
    """nodes: iterable of (prefix_k, prefix_v, len, level, batch_begin, batch_count) with the
    expanded tensors of typhoon_mla_expand_prefix.  Returns a ctypes array (host memory)."""
    arr = (tmla_prefix_node * max(1, len(nodes)))()
    for i, (k, v, ln, level, b0, bc) in enumerate(nodes):
        arr[i] = tmla_prefix_node(k.data_ptr() if k is not None else None,
                                  v.data_ptr() if v is not None else None, ln, level, b0, bc)
    return arr


def typhoon_mla_decode_tree_workspace_bytes(dims, batch, q_len, nodes, max_suffix_len):
    arr = make_nodes(nodes)
    return lib().typhoon_mla_decode_tree_workspace_bytes(ctypes.byref(dims), batch, q_len, arr,
                                                         len(nodes), max_suffix_len)


def typhoon_mla_decode_tree(dims, q, nodes, suffix_pool=None, block_table=None, suffix_lens=None,
                            max_suffix_len=0, w_uk=None, w_uv=None, out=None, lse_out=None,
                            workspace=None, want_lse=True):
    """One decode step over tree-shaped shared prefixes; returns (out, lse)."""
    B, S_q, H, _ = q.shape
    dev = q.device
    arr = make_nodes(nodes)
    if out is None:
        out = torch.empty((B, S_q, H, 128), dtype=q.dtype, device=dev)
    if lse_out is None and want_lse:
        lse_out = torch.empty((B, S_q, H), dtype=torch.float32, device=dev)
    if workspace is None:
        nbytes = lib().typhoon_mla_decode_tree_workspace_bytes(ctypes.byref(dims), B, S_q, arr,
                                                               len(nodes), max_suffix_len)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    num_blocks = suffix_pool.shape[0] if suffix_pool is not None else 0
    block_size = suffix_pool.shape[1] if suffix_pool is not None else 64
    max_blocks = block_table.shape[1] if block_table is not None else 0
    st = lib().typhoon_mla_decode_tree(
        ctypes.byref(dims), B, S_q, _ptr(q), arr, len(nodes), _ptr(suffix_pool), num_blocks,
        block_size, _ptr(block_table), max_blocks, _ptr(suffix_lens), max_suffix_len, _ptr(w_uk),
        _ptr(w_uv), _ptr(out), _ptr(lse_out), _ptr(workspace), workspace.numel(), _stream(dev))
    _check(st, "typhoon_mla_decode_tree")
    return out, lse_out
