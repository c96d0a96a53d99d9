"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad descriptors before touching HIP."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ob = pytest.importorskip("paper_2402_13720_amd.binding", reason="libouro.so not built")


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ouro.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ouro_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"ouro_verify_attn", "ouro_lmhead_argmax", "ouro_accept", "ouro_verify_attn_workspace",
            "ouro_lmhead_argmax_workspace", "ouro_lmhead_packed_w_bytes", "ouro_lmhead_pack_w", "ouro_kv_commit",
            "ouro_rope_block", "ouro_rmsnorm", "ouro_linear", "ouro_silu_mul", "ouro_fold_rmsnorm_gain",
            "ouro_interleave_gate_up", "ouro_verify_attn_plan",
            "ouro_validate_meta_host", "ouro_status_string", "ouro_last_hip_error", "ouro_version"} <= set(names)
    for n in names:
        assert hasattr(ob.lib, n), n


def test_version_and_status_strings():
    assert ob.lib.ouro_version() == 211
    assert ob.lib.ouro_status_string(0) == b"ok"
    for code in range(-9, 0):
        assert ob.lib.ouro_status_string(code) not in (b"ok", b"unknown status")
    assert ob.lib.ouro_status_string(-99) == b"unknown status"


def test_struct_sizes_match_the_header_layout():
    # 8 int32 + 7 pointers + float(+pad) + 7 pointers/size_t
    assert C.sizeof(ob.ouro_attn_desc) == 32 + 7 * 8 + 8 + 7 * 8 + 16
    assert C.sizeof(ob.ouro_lmhead_desc) == 24 + 8 * 8
    assert C.sizeof(ob.ouro_accept_desc) == 24 + 16 * 8
    assert C.sizeof(ob.ouro_kv_commit_desc) == 32 + 9 * 8 + 16


def _attn_desc(**kw):
    d = ob.ouro_attn_desc()
    d.struct_size = C.sizeof(ob.ouro_attn_desc)
    d.dtype, d.B, d.T, d.Hq, d.Hkv, d.D, d.max_seqlen = ob.OURO_BF16, 1, 64, 32, 32, 128, 2048
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_attn_descriptor_validation_runs_before_any_hip_call():
    f = ob.lib.ouro_verify_attn
    assert f(None, None) == -1
    assert f(C.byref(_attn_desc(struct_size=8)), None) == -7
    assert f(C.byref(_attn_desc(dtype=5)), None) == -3
    assert f(C.byref(_attn_desc(T=0)), None) == -2
    assert f(C.byref(_attn_desc(T=129)), None) == -2
    assert f(C.byref(_attn_desc(Hq=32, Hkv=5)), None) == -2
    assert f(C.byref(_attn_desc(D=64)), None) == -2                      # bf16 needs D = 128
    assert f(C.byref(_attn_desc(max_seqlen=-1)), None) == -2
    assert f(C.byref(_attn_desc(plan_override=-1)), None) == -2
    assert f(C.byref(_attn_desc()), None) == -1                          # data pointers are NULL
    assert f(C.byref(_attn_desc(B=0)), None) == 0                        # nothing to do
    ok = dict(q=256, k_cache=256, v_cache=256, cu_seqlens=256, k_blk=256, v_blk=256, meta=256, out=256)
    assert f(C.byref(_attn_desc(**{**ok, "q": 260})), None) == -5        # misaligned
    assert f(C.byref(_attn_desc(**ok)), None) == -1                      # workspace needed but NULL
    assert f(C.byref(_attn_desc(**ok, workspace=256, workspace_bytes=16)), None) == -4


def test_attn_workspace_query():
    ws = ob.lib.ouro_verify_attn_workspace
    assert ws(None) == 0
    assert ws(C.byref(_attn_desc(T=0))) == 0
    n = ws(C.byref(_attn_desc()))
    assert n > 0 and n % 256 == 0
    assert ws(C.byref(_attn_desc(dtype=ob.OURO_F32))) == 0
    assert ws(C.byref(_attn_desc(max_seqlen=0, T=16))) == 0              # single chunk: no partials
    assert ws(C.byref(_attn_desc(B=1, max_seqlen=65536, T=32))) > 0
    assert ws(C.byref(_attn_desc(B=16, max_seqlen=8192, T=32))) == 0    # enough sequences: one chunk each
    # a forced launch shape changes the plan, and with it the workspace: 17 chunks of 128 keys, 4 row blocks per workgroup
    forced = ws(C.byref(_attn_desc(plan_override=ob.plan_override(4, 128))))
    assert forced == 32 * 17 * 128 * (2 + 128) * 4 + (256 - 32 * 17 * 128 * 2 * 4 % 256) % 256
    assert ws(C.byref(_attn_desc(plan_override=ob.plan_override(1, 4096)))) == 0   # one chunk covers the sequence


def test_attn_launch_shape_query():
    """The host-only plan query: which kernel, keys per workgroup, chunk slots, workgroups -- on the five workloads'
    shapes and on shapes where the choice between the two bf16 kernels flips."""
    f = ob.lib.ouro_verify_attn_plan
    out = (C.c_int32 * 5)()
    assert f(None, out) == -1 and f(C.byref(_attn_desc()), None) == -1
    assert f(C.byref(_attn_desc(T=0)), out) == -2

    def plan(**kw):
        assert f(C.byref(_attn_desc(**kw)), out) == 0
        return list(out)

    assert plan() == [1, 512, 5, 320, 4]                                               # 7B layer: key-split, 5 chunks x 64 groups
    assert plan(T=128, Hq=40, Hkv=40, max_seqlen=4096) == [4, 768, 6, 240, 8]       # 13B layer: row-split (8 waves), one workgroup per CU
    assert plan(T=64, Hq=64, Hkv=8, max_seqlen=4096) == [4, 640, 7, 224, 8]         # 70B GQA layer: 16 row blocks, row-split
    assert plan(T=96, Hq=8, Hkv=8, max_seqlen=1024)[0] == 1                         # few row blocks, little K/V: key-split wins
    assert plan(B=16, T=32, max_seqlen=8192) == [1, 8320, 1, 512, 4]                # batched: one chunk (65 tiles x 4 waves) per sequence
    assert plan(B=16, T=32, Hq=64, Hkv=8, max_seqlen=4096)[0] == 4                  # GQA batch: K/V too large to re-stage per row block
    assert plan(T=128, Hq=40, Hkv=40, max_seqlen=8192)[0] == 4
    assert plan(dtype=ob.OURO_F32, T=16, Hq=4, Hkv=4, D=64, max_seqlen=128) == [0, 144, 1, 64, 0]
    assert plan(plan_override=ob.plan_override(2, 256))[:3] == [2, 256, 9]
    assert plan(T=128, Hq=40, Hkv=40, max_seqlen=4096, plan_override=ob.plan_override(4, 0, four_waves=True)) == [4, 768, 6, 240, 4]


def test_no_call_reads_the_process_environment(monkeypatch):
    """Tuning goes through descriptor fields; environment variables of the earlier interface are ignored."""
    ws = ob.lib.ouro_verify_attn_workspace
    before = ws(C.byref(_attn_desc()))
    monkeypatch.setenv("OURO_ATTN_CHUNK", "128")
    monkeypatch.setenv("OURO_ATTN_RW", "4")
    monkeypatch.setenv("OURO_LINEAR_KSPLIT", "7")
    assert ws(C.byref(_attn_desc())) == before
    d = ob.ouro_linear_desc()
    d.struct_size = C.sizeof(ob.ouro_linear_desc)
    d.dtype, d.R, d.K, d.N = ob.OURO_BF16, 64, 4096, 4096
    auto = ob.lib.ouro_linear_workspace(C.byref(d))
    assert auto == 8 * 64 * (4096 + 1) * 4                                # the heuristic: 32 slabs -> 8 shares of the k range
    d.ksplit_override = 3
    assert ob.lib.ouro_linear_workspace(C.byref(d)) == 3 * 64 * (4096 + 1) * 4
    d.ksplit_override = -1
    assert ob.lib.ouro_linear_workspace(C.byref(d)) == 0 and ob.lib.ouro_linear(C.byref(d), None) == -2


def test_weight_relayout_validation():
    for f in (ob.lib.ouro_fold_rmsnorm_gain, ob.lib.ouro_interleave_gate_up):
        assert f(None, 256, 512, 8, 64, None) == -1
        assert f(256, 512, 1024, 0, 64, None) == -2
        assert f(256, 512, 1024, 8, 60, None) == -2                       # K must be a multiple of 8
        assert f(256, 520, 1024, 8, 64, None) == -5


def _lm_desc(**kw):
    d = ob.ouro_lmhead_desc()
    d.struct_size = C.sizeof(ob.ouro_lmhead_desc)
    d.dtype, d.R, d.Hd, d.V = ob.OURO_BF16, 64, 4096, 32000
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_lmhead_descriptor_validation():
    f = ob.lib.ouro_lmhead_argmax
    assert f(None, None) == -1
    assert f(C.byref(_lm_desc(struct_size=4)), None) == -7
    assert f(C.byref(_lm_desc(dtype=2)), None) == -3
    assert f(C.byref(_lm_desc(Hd=4000 + 8)), None) == -2                 # bf16: Hd multiple of 64
    assert f(C.byref(_lm_desc(V=0)), None) == -2
    assert f(C.byref(_lm_desc(R=0)), None) == 0
    assert f(C.byref(_lm_desc()), None) == -1
    ok = dict(hidden=512, w=512, argmax_out=512)
    assert f(C.byref(_lm_desc(**ok)), None) == -1                        # workspace NULL
    assert f(C.byref(_lm_desc(**ok, workspace=512, workspace_bytes=8)), None) == -4
    need = ob.lib.ouro_lmhead_argmax_workspace(C.byref(_lm_desc()))
    assert need >= 250 * 64 * 8


def test_static_scratch_entry_point_rejects_what_its_buffer_cannot_hold():
    """ouro_lmhead_argmax_static needs no workspace; sizes beyond its built-in 2 MiB are refused before any HIP call."""
    f = ob.lib.ouro_lmhead_argmax_static
    assert f(None, None) == -1
    assert f(C.byref(_lm_desc(struct_size=4)), None) == -7
    assert f(C.byref(_lm_desc(V=0)), None) == -2
    assert f(C.byref(_lm_desc()), None) == -1                                       # data pointers missing
    assert f(C.byref(_lm_desc(R=0)), None) == 0
    ok = dict(hidden=512, w=512, argmax_out=512)
    need = lambda **kw: ob.lib.ouro_lmhead_argmax_workspace(C.byref(_lm_desc(**kw)))
    assert need(R=2097) <= (2 << 20) < need(R=2098)
    assert f(C.byref(_lm_desc(R=2098, **ok)), None) == -9                           # 125 slabs x 2098 rows x 8 bytes > 2 MiB
    assert f(C.byref(_lm_desc(R=64, V=5_000_000, **ok)), None) == -9
    assert ob.lib.ouro_status_string(-9) not in (b"ok", b"unknown status")


def test_packed_weight_helpers():
    f = ob.lib.ouro_lmhead_packed_w_bytes
    assert f(32000, 4096) == 32000 * 4096 * 2
    assert f(1000, 256) == 1024 * 256 * 2            # rows padded to a multiple of 128
    assert f(0, 64) == 0 and f(10, 100) == 0
    g = ob.lib.ouro_lmhead_pack_w
    assert g(None, 256, 10, 64, None) == -1
    assert g(256, 512, 10, 100, None) == -2
    assert g(260, 512, 10, 64, None) == -5
    lm = ob.lib.ouro_lmhead_argmax
    assert lm(C.byref(_lm_desc(w_layout=7)), None) == -2
    assert lm(C.byref(_lm_desc(w_layout=1, dtype=ob.OURO_F32)), None) == -2


def _acc_desc(**kw):
    d = ob.ouro_accept_desc()
    d.struct_size = C.sizeof(ob.ouro_accept_desc)
    d.B, d.T, d.gamma, d.K, d.beta = 1, 64, 16, 8, 6
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_accept_descriptor_validation():
    f = ob.lib.ouro_accept
    assert f(None, None) == -1
    assert f(C.byref(_acc_desc(struct_size=1)), None) == -7
    assert f(C.byref(_acc_desc(T=63)), None) == -2                       # T != gamma + K*beta
    assert f(C.byref(_acc_desc(gamma=0, T=48)), None) == -2
    assert f(C.byref(_acc_desc(K=64, beta=1, gamma=64, T=128)), None) == -2
    assert f(C.byref(_acc_desc()), None) == -1
    p = 4096
    need = dict(draft_tok=p, argmax=p, meta=p, n_accept=p, path=p, bonus=p, accept_idx=p)
    assert f(C.byref(_acc_desc(**need, n_seg=p)), None) == -1            # segment outputs: all three or none
    assert f(C.byref(_acc_desc(B=0)), None) == 0


def _commit_desc(**kw):
    d = ob.ouro_kv_commit_desc()
    d.struct_size = C.sizeof(ob.ouro_kv_commit_desc)
    d.dtype = ob.OURO_BF16
    d.B, d.T, d.Hkv, d.D, d.max_accept = 1, 64, 32, 128, 22
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_kv_commit_descriptor_validation():
    f = ob.lib.ouro_kv_commit
    assert f(None, None) == -1
    assert f(C.byref(_commit_desc(struct_size=3)), None) == -7
    assert f(C.byref(_commit_desc(dtype=5)), None) == -3
    assert f(C.byref(_commit_desc(max_accept=0)), None) == -2
    assert f(C.byref(_commit_desc(max_accept=65)), None) == -2            # more slots than block tokens
    assert f(C.byref(_commit_desc(Hkv=1, D=4)), None) == -2               # 8-byte rows: not a multiple of 16
    assert f(C.byref(_commit_desc()), None) == -1                         # pointers missing
    p = 4096
    full = dict(k_blk=p, v_blk=p, accept_idx=p, n_accept=p, k_cache=p, v_cache=p, cu_seqlens=p, seq_len=p, overflow=p)
    assert f(C.byref(_commit_desc(**{**full, "k_cache": p + 8})), None) == -5
    assert f(C.byref(_commit_desc(B=0)), None) == 0


def test_layer_descriptor_validation():
    for name, desc in (("ouro_rope_block", ob.ouro_rope_desc), ("ouro_rmsnorm", ob.ouro_rmsnorm_desc),
                       ("ouro_linear", ob.ouro_linear_desc), ("ouro_silu_mul", ob.ouro_silu_mul_desc)):
        f = getattr(ob.lib, name)
        assert f(None, None) == -1
        d = desc()
        d.struct_size = 4
        assert f(C.byref(d), None) == -7
    d = ob.ouro_linear_desc()
    d.struct_size = C.sizeof(ob.ouro_linear_desc)
    d.dtype, d.R, d.K, d.N = ob.OURO_F32, 4, 64, 8
    assert ob.lib.ouro_linear(C.byref(d), None) == -3                     # bf16 only
    d.dtype, d.K = ob.OURO_BF16, 100
    assert ob.lib.ouro_linear(C.byref(d), None) == -2                     # K must be a multiple of 64
    d.K, d.N = 64, 12
    assert ob.lib.ouro_linear(C.byref(d), None) == -2                     # N must be a multiple of 8
    d.N, d.epilogue = 8, ob.OURO_EPI_SWIGLU_PAIRS
    assert ob.lib.ouro_linear(C.byref(d), None) == -2                     # gated form: N must be a multiple of 16
    d.epilogue = 7
    assert ob.lib.ouro_linear(C.byref(d), None) == -2                     # unknown epilogue
    d.epilogue = ob.OURO_EPI_NONE
    assert C.sizeof(ob.ouro_linear_desc) == 40 + 5 * 8 + 8
    assert ob.lib.ouro_linear(C.byref(d), None) == -1                     # pointers missing
    d.R = 0
    assert ob.lib.ouro_linear(C.byref(d), None) == 0
    r = ob.ouro_rope_desc()
    r.struct_size = C.sizeof(ob.ouro_rope_desc)
    r.dtype, r.B, r.T, r.Hq, r.Hkv, r.D = ob.OURO_BF16, 1, 8, 2, 2, 7
    assert ob.lib.ouro_rope_block(C.byref(r), None) == -2                 # odd head dim
    r.D = 8
    assert ob.lib.ouro_rope_block(C.byref(r), None) == -1
    assert C.sizeof(ob.ouro_rope_desc) == 32 + 8 * 8                      # 8 ints/floats, 8 pointers


def test_validate_meta_host():
    from paper_2402_13720_amd import workloads as W
    cfg = W.CONFIGS[2]
    pid, boff = W.make_block_meta(cfg, np.random.default_rng(0))
    meta = np.stack([pid[0], boff[0]], axis=-1).astype(np.int16).copy()
    f = ob.lib.ouro_validate_meta_host
    p = meta.ctypes.data_as(C.c_void_p)
    assert f(p, cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == 0
    assert f(None, cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == -1
    assert f(p, cfg.T + 1, cfg.gamma, cfg.K, cfg.beta_p) == -2
    bad = meta.copy(); bad[3, 1] = 2                                     # main token with wrong branch_off
    assert f(bad.ctypes.data_as(C.c_void_p), cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == -8
    bad = meta.copy(); bad[cfg.gamma + 1, 0] = 5                         # phrase id broken inside a phrase
    assert f(bad.ctypes.data_as(C.c_void_p), cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == -8
    bad = meta.copy(); bad[cfg.gamma:cfg.gamma + cfg.beta_p, 1] = cfg.gamma   # branch beyond the main draft
    assert f(bad.ctypes.data_as(C.c_void_p), cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == -8
    ok = meta.copy(); ok[cfg.gamma:cfg.gamma + cfg.beta_p, 1] = -1       # phrase hanging off the prefix
    assert f(ok.ctypes.data_as(C.c_void_p), cfg.T, cfg.gamma, cfg.K, cfg.beta_p) == 0
