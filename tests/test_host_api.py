"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, validates its
arguments on the host (no launch happens on an error path) and sizes its buffers sensibly."""
import ctypes
import os
import re

import pytest

from paper_2509_21081_amd import binding as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _dims(**kw):
    d = dict(num_heads=16, sm_scale=0.07, dtype=T.BF16)
    d.update(kw)
    return T.make_dims(**d)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "typhoon_mla.h")).read()
    declared = set(re.findall(r"\b(typhoon_mla_\w+)\s*\(", header))
    assert declared == set(T.EXPORTS)
    L = T.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    assert T.typhoon_mla_status_string(0) == "ok"
    for s in range(1, 6):
        assert T.typhoon_mla_status_string(s) not in ("ok", "unknown status")
    assert T.typhoon_mla_status_string(99) == "unknown status"


def test_expanded_sizes():
    d = _dims(num_heads=128)
    # bf16: 640 bytes per token-head, tokens padded to 32 (Table 1: L_s H (D_qk + D_v) words)
    assert T.typhoon_mla_expanded_k_bytes(d, 4096) == 128 * 4096 * 192 * 2
    assert T.typhoon_mla_expanded_v_bytes(d, 4096) == 128 * 4096 * 128 * 2
    assert T.typhoon_mla_expanded_k_bytes(d, 33) == 128 * 64 * 192 * 2
    f = _dims(num_heads=16, dtype=T.FP32)
    assert T.typhoon_mla_expanded_k_bytes(f, 33) == 16 * 33 * 192 * 4
    assert T.typhoon_mla_expanded_k_bytes(_dims(kv_lora_rank=256), 10) == 0


def test_dims_validation():
    L = T.lib()
    P = ctypes.byref
    nul = ctypes.c_void_p(None)
    one = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    assert L.typhoon_mla_expand_prefix(None, 4, one, one, one, one, one, one, nul) == \
        T.TMLA_ERR_INVALID_ARG
    for bad in (dict(kv_lora_rank=256), dict(qk_nope_dim=64), dict(num_heads=24), dict(dtype=7)):
        assert L.typhoon_mla_expand_prefix(P(_dims(**bad)), 4, one, one, one, one, one, one, nul) \
            == T.TMLA_ERR_UNSUPPORTED, bad
    assert L.typhoon_mla_expand_prefix(P(_dims(num_heads=0)), 4, one, one, one, one, one, one,
                                       nul) == T.TMLA_ERR_INVALID_ARG
    assert L.typhoon_mla_expand_prefix(P(_dims(sm_scale=-1.0)), 4, one, one, one, one, one, one,
                                       nul) == T.TMLA_ERR_INVALID_ARG
    d = _dims()
    assert L.typhoon_mla_expand_prefix(P(d), -1, one, one, one, one, one, one, nul) == \
        T.TMLA_ERR_INVALID_ARG
    assert L.typhoon_mla_expand_prefix(P(d), 4, nul, one, one, one, one, one, nul) == \
        T.TMLA_ERR_INVALID_ARG
    assert L.typhoon_mla_expand_prefix(P(d), 4, ctypes.c_void_p(4100), one, one, one, one, one,
                                       nul) == T.TMLA_ERR_INVALID_ARG        # misaligned
    assert L.typhoon_mla_expand_prefix(P(d), 0, nul, nul, nul, nul, nul, nul, nul) == T.TMLA_OK
    assert L.typhoon_mla_expand_pool(P(d), 3, 48, one, one, one, one, one, nul) == \
        T.TMLA_ERR_UNSUPPORTED


def _decode(L, d, mode=0, batch=2, q_len=1, prefix_len=64, max_suffix=100, block_size=64,
            max_blocks=2, ws_bytes=None, **ptr_overrides):
    one = ctypes.c_void_p(4096)
    names = ["q", "prefix_k", "prefix_v", "prefix_ckv", "prefix_krope", "suffix_pool",
             "block_table", "suffix_lens", "suffix_k_pool", "suffix_v_pool", "w_uk", "w_uv", "out",
             "lse_out", "workspace"]
    p = {n: one for n in names}
    for k, v in ptr_overrides.items():
        p[k] = ctypes.c_void_p(v)
    if ws_bytes is None:
        ws_bytes = T.typhoon_mla_decode_workspace_bytes(d, mode, batch, q_len, prefix_len,
                                                        max_suffix)
    return L.typhoon_mla_decode(
        ctypes.byref(d), mode, batch, q_len, p["q"], prefix_len, p["prefix_k"], p["prefix_v"],
        p["prefix_ckv"], p["prefix_krope"], p["suffix_pool"], 8, block_size, p["block_table"],
        max_blocks, p["suffix_lens"], max_suffix, p["suffix_k_pool"], p["suffix_v_pool"],
        p["w_uk"], p["w_uv"], p["out"], p["lse_out"], p["workspace"], ws_bytes, None)


def test_decode_validation_without_gpu():
    L = T.lib()
    d = _dims()
    assert _decode(L, d, mode=5) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, q_len=0) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, q_len=9) == T.TMLA_ERR_UNSUPPORTED
    assert _decode(L, d, prefix_len=(1 << 30) + 1, ws_bytes=1 << 20) == T.TMLA_ERR_UNSUPPORTED
    assert _decode(L, d, batch=-1) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, prefix_len=-3) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, block_size=32) == T.TMLA_ERR_UNSUPPORTED
    assert _decode(L, d, max_suffix=200, max_blocks=2) == T.TMLA_ERR_INVALID_ARG  # 2*64 < 200
    assert _decode(L, d, q=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, out=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, suffix_lens=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, prefix_k=None) == T.TMLA_ERR_INVALID_ARG                # mixed needs it
    assert _decode(L, d, mode=2, prefix_ckv=None) == T.TMLA_ERR_INVALID_ARG      # absorb_only
    assert _decode(L, d, mode=1, suffix_k_pool=None) == T.TMLA_ERR_INVALID_ARG   # naive_only
    assert _decode(L, d, suffix_pool=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, w_uk=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, q=4104) == T.TMLA_ERR_INVALID_ARG                        # misaligned
    assert _decode(L, d, workspace=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, workspace=4096 + 64) == T.TMLA_ERR_INVALID_ARG           # needs 256 B
    assert _decode(L, d, ws_bytes=128) == T.TMLA_ERR_WORKSPACE_TOO_SMALL
    assert _decode(L, d, batch=0) == T.TMLA_OK                                    # nothing to do


def test_workspace_bytes_monotone_and_zero_on_error():
    d = _dims(num_heads=128)
    assert T.typhoon_mla_decode_workspace_bytes(d, 7, 4, 1, 10, 10) == 0
    assert T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 1, 1, 2_000_000_000, 10) == 0
    assert T.typhoon_mla_decode_workspace_bytes(d, T.MODE_ABSORB_ONLY, 1, 1, 1 << 30, 1 << 30) > 0
    small = T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 4, 1, 256, 64)
    big = T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 64, 1, 4096, 512)
    assert 0 < small < big
    # the absorbed queries alone need B*S_q*H*576 elements
    assert big >= 64 * 128 * 576 * 2


def test_tuning_overrides_change_the_plan_and_are_restored():
    d = _dims(num_heads=128)
    L = T.lib()
    assert L.typhoon_mla_set_tuning(99, 1) == -1 and L.typhoon_mla_set_tuning(-1, 1) == -1
    assert L.typhoon_mla_set_tuning(T.TUNE_SUFFIX_CHUNK, -5) == -1
    base = T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 64, 1, 4096, 2048)
    old = T.typhoon_mla_set_tuning(T.TUNE_SUFFIX_CHUNK, 64)
    try:
        # 32 chunks of 64 tokens per request instead of a few long ones: more latent partials
        assert T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 64, 1, 4096, 2048) > base
        assert T.typhoon_mla_set_tuning(T.TUNE_SUFFIX_CHUNK, old) == 64
    finally:
        T.typhoon_mla_set_tuning(T.TUNE_SUFFIX_CHUNK, old)
    assert T.typhoon_mla_decode_workspace_bytes(d, T.MODE_MIXED, 64, 1, 4096, 2048) == base


def test_static_scratch_decode_validates_before_touching_the_gpu():
    """Same argument checks as typhoon_mla_decode, and a clear error for a problem whose
    intermediates do not fit the static array -- all on the host, nothing launched."""
    L = T.lib()
    P = ctypes.byref
    p4k = ctypes.c_void_p(4096)

    def call(d, batch=4, mode=0, q=p4k, prefix_len=256, max_suffix=100, max_blocks=2,
             block_size=64, num_blocks=9):
        return L.typhoon_mla_decode_static_scratch(
            P(d), mode, batch, 1, q, prefix_len, p4k, p4k, p4k, p4k, p4k, num_blocks, block_size,
            p4k, max_blocks, p4k, max_suffix, None, None, p4k, p4k, p4k, None, None)
    d = _dims(num_heads=128)
    assert call(d, q=None) == T.TMLA_ERR_INVALID_ARG
    assert call(d, mode=7) == T.TMLA_ERR_INVALID_ARG
    assert call(d, block_size=48) == T.TMLA_ERR_UNSUPPORTED
    assert call(d, max_suffix=200) == T.TMLA_ERR_INVALID_ARG            # 2*64 < 200
    assert call(d, batch=0) == T.TMLA_OK
    assert T.typhoon_mla_decode_workspace_bytes(d, 0, 2048, 1, 4096, 4096) > T.STATIC_SCRATCH_BYTES
    assert call(d, batch=2048, prefix_len=4096, max_suffix=4096, max_blocks=64) == \
        T.TMLA_ERR_SCRATCH_LIMIT
    assert "static" in T.typhoon_mla_status_string(T.TMLA_ERR_SCRATCH_LIMIT)
    header = open(os.path.join(ROOT, "include", "typhoon_mla.h")).read()
    assert "#define TMLA_STATIC_SCRATCH_BYTES (128u << 20)" in header
    # the benchmark configurations all fit
    for B, S, H, Ls, Ln in [(64, 1, 128, 4096, 512), (256, 1, 128, 32768, 2048),
                            (128, 2, 128, 8192, 1024), (512, 1, 16, 16384, 4096)]:
        dd = _dims(num_heads=H)
        for m in (T.MODE_MIXED, T.MODE_ABSORB_ONLY, T.MODE_NAIVE_ONLY):
            assert T.typhoon_mla_decode_workspace_bytes(dd, m, B, S, Ls, Ln) <= T.STATIC_SCRATCH_BYTES


def test_combine_validation():
    L = T.lib()
    one = ctypes.c_void_p(4096)
    assert L.typhoon_mla_combine_lse(0, 4, 128, one, one, one, 1, None, None) == \
        T.TMLA_ERR_INVALID_ARG
    assert L.typhoon_mla_combine_lse(2, 4, 130, one, one, one, 1, None, None) == \
        T.TMLA_ERR_UNSUPPORTED
    assert L.typhoon_mla_combine_lse(2, 4, 1024, one, one, one, 1, None, None) == \
        T.TMLA_ERR_UNSUPPORTED
    assert L.typhoon_mla_combine_lse(2, 4, 128, None, one, one, 1, None, None) == \
        T.TMLA_ERR_INVALID_ARG
    assert L.typhoon_mla_combine_lse(2, 0, 128, None, None, None, 1, None, None) == T.TMLA_OK


def test_auto_mode_threshold_follows_break_even_formula():
    from paper_2509_21081_amd import cost_model as C
    d128, d64, d16 = _dims(num_heads=128), _dims(num_heads=64), _dims(num_heads=16)
    thr = T.typhoon_mla_auto_batch_threshold
    # the measured cross-overs the table holds (mixed overtakes absorb_only at this batch)
    assert abs(thr(d128, 1, 4096) - 45) < 1e-9 and abs(thr(d128, 1, 16384) - 40) < 1e-9
    assert abs(thr(d64, 1, 16384) - 35) < 1e-9 and abs(thr(d16, 1, 65536) - 11) < 1e-9
    assert abs(thr(d64, 1, 1024) - 128) < 1e-9
    # clamped outside the table, interpolated geometrically inside
    assert thr(d128, 1, 100) == thr(d128, 1, 1024) and thr(d128, 1, 1 << 20) == thr(d128, 1, 65536)
    assert thr(_dims(num_heads=256), 1, 16384) == thr(d128, 1, 16384)
    assert abs(thr(d128, 1, 8192) - (thr(d128, 1, 4096) * thr(d128, 1, 16384)) ** 0.5) < 1e-9
    d32 = _dims(num_heads=32)
    assert abs(thr(d32, 1, 2048) - 32) < 1e-9          # sqrt(64 * 16)
    # Section 3.2: the break-even batch falls as 1 / S_q
    assert abs(thr(d128, 2, 4096) - thr(d128, 1, 4096) / 2) < 1e-9
    # in the paper's form: the same closed formula with the effective absorb throughput that this
    # threshold implies against the naive pass's 5.5 TB/s
    t_eff = thr(d128, 1, 16384) * 5.5e12 * (2 * 512 + 64) / (192 + 128)
    assert abs(C.batch_threshold(t_eff, 5.5e12, 1) - thr(d128, 1, 16384)) < 1e-9
    assert 300e12 < t_eff < 1500e12
    assert thr(_dims(kv_lora_rank=256), 1, 4096) == -1
    L = T.lib()
    d = _dims()
    # auto needs both forms of the prefix
    assert _decode(L, d, mode=3, prefix_ckv=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, mode=3, prefix_k=None) == T.TMLA_ERR_INVALID_ARG
    assert _decode(L, d, mode=4) == T.TMLA_ERR_INVALID_ARG
    big = T.typhoon_mla_decode_workspace_bytes(d128, T.MODE_AUTO, 64, 1, 4096, 512)
    assert big == T.typhoon_mla_decode_workspace_bytes(d128, T.MODE_MIXED, 64, 1, 4096, 512)
    small = T.typhoon_mla_decode_workspace_bytes(d128, T.MODE_AUTO, 1, 1, 4096, 512)
    assert small == T.typhoon_mla_decode_workspace_bytes(d128, T.MODE_ABSORB_ONLY, 1, 1, 4096, 512)


def test_tree_decode_validation():
    import ctypes
    L = T.lib()
    d = _dims()
    nul = ctypes.c_void_p(None)
    one = ctypes.c_void_p(4096)   # never dereferenced: every case below fails validation first

    def call(nodes, batch=4, q=one, ws=one, ws_bytes=1 << 30, block_size=64):
        arr = T.make_nodes(nodes)
        return L.typhoon_mla_decode_tree(ctypes.byref(d), batch, 1, q, arr, len(nodes), nul, 0,
                                         block_size, nul, 0, one, 0, nul, nul, one, nul, ws,
                                         ws_bytes, nul)

    class P:   # stands in for a device tensor
        def __init__(self, addr): self.addr = addr
        def data_ptr(self): return self.addr
    k = P(4096)
    ok_nodes = [(k, k, 100, 0, 0, 4), (k, k, 50, 1, 0, 2), (k, k, 60, 1, 2, 2)]
    assert T.typhoon_mla_decode_tree_workspace_bytes(d, 4, 1, ok_nodes, 0) > 0
    assert call([], batch=0) == T.TMLA_OK                          # nothing to do
    assert call(ok_nodes, batch=0) == T.TMLA_ERR_INVALID_ARG       # nodes outside the batch
    assert call(ok_nodes, q=nul) == T.TMLA_ERR_INVALID_ARG
    assert call(ok_nodes, ws_bytes=16) == T.TMLA_ERR_WORKSPACE_TOO_SMALL
    assert call(ok_nodes, block_size=48) == T.TMLA_ERR_UNSUPPORTED
    assert call([(k, k, 100, 0, 0, 4), (k, k, 50, 0, 3, 1)]) == T.TMLA_ERR_INVALID_ARG   # overlap
    assert call([(k, k, 100, 8, 0, 4)]) == T.TMLA_ERR_INVALID_ARG                        # level
    assert call([(k, k, 100, 0, 2, 3)]) == T.TMLA_ERR_INVALID_ARG                        # range
    assert call([(k, k, -1, 0, 0, 4)]) == T.TMLA_ERR_INVALID_ARG
    assert call([(None, None, 100, 0, 0, 4)]) == T.TMLA_ERR_INVALID_ARG                  # no K/V
    assert call([(P(4100), k, 100, 0, 0, 4)]) == T.TMLA_ERR_INVALID_ARG                  # misaligned
    # more levels need more partial slots
    w1 = T.typhoon_mla_decode_tree_workspace_bytes(d, 4, 1, ok_nodes[:1], 64)
    w2 = T.typhoon_mla_decode_tree_workspace_bytes(d, 4, 1, ok_nodes, 64)
    assert 0 < w1 < w2
