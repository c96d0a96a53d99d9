"""GPU parity: ouro_verify_attn (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W
from gpu_util import DEV, attn_tol, run_attention, to_np64

pytestmark = pytest.mark.gpu


def _oracle(inp, heads=None):
    return O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                              inp["pid"], inp["boff"], heads=heads)


def _check(cfg, inp, heads=None, lse_tol=None, head_major=False, rw=0, chunk=0):
    out, lse, _ = run_attention(cfg, inp, head_major=head_major, rw=rw, chunk=chunk)
    ref = _oracle(inp, heads)
    got = to_np64(out)
    got_lse = to_np64(lse)
    assert np.isfinite(got).all()
    if heads is None:
        err = np.abs(got - ref["out"]).max()
        lerr = np.abs(got_lse - ref["lse"]).max()
    else:
        err = max(np.abs(got[b, :, h] - ref["out"][b, :, h]).max() for b, h in heads)
        lerr = max(np.abs(got_lse[b, h] - ref["lse"][b, h]).max() for b, h in heads)
    print("%s: max-abs err %.3g, lse err %.3g" % (cfg.name, err, lerr), flush=True)
    assert err <= attn_tol(cfg), err
    assert lerr <= (lse_tol or (1e-2 if cfg.dtype == "bf16" else 1e-5)), lerr
    return out


def test_config1_fp32_tiny():
    cfg = W.CONFIGS[1]
    for trial in range(3):
        _check(cfg, W.make_attention_inputs(cfg, W.seed_for(1, trial)))


@pytest.mark.parametrize("kw", [
    dict(D=128, Hq=4, Hkv=2, B=3, L=(0, 70)),
    dict(D=64, Hq=6, Hkv=1, B=2, L=(60, 130), gamma=5, K=3, beta_p=7),
    dict(D=64, B=2, L=(0, 0)),
    dict(D=128, gamma=9, K=0, beta_p=0, L=33),
])
def test_fp32_shapes(kw):
    cfg = W.scaled(W.CONFIGS[1], **kw)
    _check(cfg, W.make_attention_inputs(cfg, 77))


@pytest.mark.parametrize("kw", [
    dict(B=2, Hq=4, Hkv=2, L=(0, 300), gamma=10, K=5, beta_p=6),        # 80 rows per KV head: 2 row blocks, ragged
    dict(B=3, Hq=2, Hkv=2, L=(1, 200), gamma=3, K=2, beta_p=4),         # 11 rows: one partially filled tile
    dict(B=1, Hq=8, Hkv=1, L=517, gamma=16, K=8, beta_p=6),             # GQA 8: 512 rows, 8 row blocks
    dict(B=2, Hq=2, Hkv=2, L=(0, 0), gamma=8, K=4, beta_p=6),           # empty cache
    dict(B=1, Hq=2, Hkv=2, L=1000, gamma=32, K=16, beta_p=6),           # T = 128
    dict(B=4, Hq=2, Hkv=1, L=(30, 2000), gamma=8, K=4, beta_p=6),       # very uneven lengths
    dict(B=1, Hq=1, Hkv=1, L=95, gamma=1, K=0, beta_p=0),               # a single row
])
@pytest.mark.parametrize("branch", ["uniform", "last"])
def test_bf16_small_shapes(kw, branch):
    cfg = W.scaled(W.CONFIGS[2], **kw)
    _check(cfg, W.make_attention_inputs(cfg, 1234, branch=branch))


@pytest.mark.parametrize("head_major", [False, True])
@pytest.mark.parametrize("rw", [1, 2, 4, 4 + 0x80])
@pytest.mark.parametrize("kw, chunk", [
    (dict(B=2, Hq=4, Hkv=2, L=(0, 300), gamma=10, K=5, beta_p=6), 0),         # 80 rows; one sequence is all block
    (dict(B=1, Hq=8, Hkv=1, L=517, gamma=16, K=8, beta_p=6), 128),            # GQA 8: 512 rows; 5 one-stage chunks
    (dict(B=1, Hq=2, Hkv=2, L=1000, gamma=32, K=16, beta_p=6), 384),          # T = 128; 3 stages per chunk, ragged
    (dict(B=4, Hq=2, Hkv=1, L=(30, 2000), gamma=8, K=4, beta_p=6), 512),      # uneven lengths, empty chunk slots
    (dict(B=1, Hq=1, Hkv=1, L=95, gamma=1, K=0, beta_p=0), 0),                # a single row
])
def test_bf16_every_kernel_variant(kw, chunk, rw, head_major):
    """The launch heuristic picks the row blocks per workgroup (1: waves split the keys; 2, 4: waves split the
    rows and share staged tiles: 4 is the eight-wave kernel with two key groups per row block, 4 + 0x80 the
    four-wave one) and the chunk length; force each combination so that every kernel sees several stages, several chunks and a ragged
    tail, with the cache in either layout."""
    cfg = W.scaled(W.CONFIGS[2], **kw)
    _check(cfg, W.make_attention_inputs(cfg, 4321), head_major=head_major, rw=rw, chunk=chunk)


def test_fp32_head_major_cache():
    cfg = W.scaled(W.CONFIGS[1], B=3, L=(0, 300))
    _check(cfg, W.make_attention_inputs(cfg, 78), head_major=True)


def test_bf16_phrase_hanging_off_the_prefix():
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=2, Hkv=2, L=70, gamma=4, K=3, beta_p=5)
    inp = W.make_attention_inputs(cfg, 5)
    inp["boff"][0, cfg.gamma:cfg.gamma + cfg.beta_p] = -1
    _check(cfg, inp)


def test_bf16_max_seqlen_hint_may_exceed_actual_lengths():
    cfg = W.scaled(W.CONFIGS[2], B=2, Hq=2, Hkv=2, L=(10, 100))
    inp = W.make_attention_inputs(cfg, 6)
    a, _, _ = run_attention(cfg, inp)
    b, _, _ = run_attention(cfg, inp, max_seqlen=4096)
    ref = _oracle(inp)["out"]
    assert np.abs(to_np64(a) - ref).max() <= 2e-2 and np.abs(to_np64(b) - ref).max() <= 2e-2


def test_bf16_mask_probe_through_the_kernel():
    """Q = 0 and V = one-hot(key index): output * (number of visible keys) is the mask row (closed form)."""
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=1, Hkv=1, L=64, gamma=16, K=8, beta_p=6)
    inp = W.make_attention_inputs(cfg, 8)
    inp["q"][:] = 0
    eye = np.eye(128, dtype=np.float32)
    inp["v_cache"] = eye[:64, None, :].copy()
    inp["v_blk"] = eye[None, 64:, None, :].copy()
    out, lse, _ = run_attention(cfg, inp)
    nvis = np.exp(to_np64(lse)[0, 0])                     # scores are all zero: lse = log(#visible)
    rec = np.rint(to_np64(out)[0, :, 0, :] * nvis[:, None])
    want = O.dense_mask(inp["pid"][0], inp["boff"][0], 64).astype(float)
    assert np.array_equal(rec, want)
    assert np.allclose(nvis, want.sum(1), atol=1e-3)


@pytest.mark.parametrize("head_major", [False, True])
@pytest.mark.parametrize("cfg_id", [2, 3, 4, 5])
def test_full_size_configs_every_head_and_row(cfg_id, head_major):
    """Every output element of the workload at its full size against the oracle (no sampling), in both cache layouts,
    in the launch configuration the benchmark times; plus run-to-run determinism (fixed merge order, no float atomics)."""
    from gpu_util import full_size_attention_case
    cfg = W.CONFIGS[cfg_id]
    inp, ref = full_size_attention_case(cfg_id)
    out, lse, _ = run_attention(cfg, inp, head_major=head_major)
    got, got_lse = to_np64(out), to_np64(lse)
    assert np.isfinite(got).all()
    err, lerr = np.abs(got - ref["out"]).max(), np.abs(got_lse - ref["lse"]).max()
    print("%s: %d x %d x %d rows, max-abs err %.3g, lse err %.3g" % (cfg.name, cfg.B, cfg.T, cfg.Hq, err, lerr), flush=True)
    assert err <= attn_tol(cfg) and lerr <= 1e-2
    out2, _, _ = run_attention(cfg, inp, head_major=head_major)
    assert torch.equal(out, out2)


@pytest.mark.parametrize("cfg_id, kw, rw", [
    (2, dict(B=3, Hq=4, Hkv=2, L=(300, 1500)), 1),               # key-split kernel; the hint cuts chunk slots away
    (2, dict(B=2, Hq=16, Hkv=2, L=(300, 1500)), 4),              # row-split kernel
    (2, dict(B=2, Hq=16, Hkv=2, L=(300, 1500)), 4 + 0x80),       # row-split kernel, four waves
    (1, dict(B=2, L=(100, 300)), 0),                             # fp32 kernel
])
def test_length_beyond_the_hint_is_cut_to_the_hint(cfg_id, kw, rw):
    """max_seqlen sizes the grid, the chunk slots and the workspace.  A device-side length above it (a stale hint: the
    commit advances lengths on the device) must not reach past any of them: such a sequence is attended over its first
    max_seqlen cached tokens, which is what the oracle computes when told that length."""
    cfg = W.scaled(W.CONFIGS[cfg_id], **kw)
    inp = W.make_attention_inputs(cfg, 31 + cfg_id)
    lens = np.diff(inp["cu_seqlens"])
    hint = int(lens.min()) + 7                                                 # below the longest sequence
    assert lens.max() > hint
    out, lse, _ = run_attention(cfg, inp, max_seqlen=hint, rw=rw)
    ref = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                             inp["pid"], inp["boff"], seq_len=np.minimum(lens, hint))
    assert np.abs(to_np64(out) - ref["out"]).max() <= attn_tol(cfg)
    assert np.abs(to_np64(lse) - ref["lse"]).max() <= (1e-2 if cfg.dtype == "bf16" else 1e-5)


def test_workspace_is_reusable_across_shapes_and_calls():
    """A workspace may hold anything on entry and can be shared by calls of different shapes."""
    from paper_2402_13720_amd import binding as ob
    from gpu_util import upload_attention
    ws = torch.full((64 << 20,), 0xA5, dtype=torch.uint8, device=DEV)
    for kw, seed in [(dict(B=2, Hq=4, Hkv=2, L=(700, 3000)), 1), (dict(B=1, Hq=8, Hkv=8, L=5000), 2),
                     (dict(B=2, Hq=4, Hkv=2, L=(700, 3000)), 1)]:
        cfg = W.scaled(W.CONFIGS[2], **kw)
        inp = W.make_attention_inputs(cfg, seed)
        t = upload_attention(cfg, inp)
        assert ob.ouro_verify_attn_workspace(t["q"], t["k_blk"], t["max_seqlen"]) <= ws.numel()
        ref = _oracle(inp)["out"]
        for _ in range(2):
            out = ob.ouro_verify_attn(t["q"], t["k_cache"], t["v_cache"], t["cu_seqlens"], t["k_blk"], t["v_blk"],
                                      t["meta"], t["max_seqlen"], workspace=ws)
            torch.cuda.synchronize()
            assert np.abs(to_np64(out) - ref).max() <= 2e-2


@pytest.mark.parametrize("cfg_id, kw", [
    (1, dict(B=2, L=(0, 300))),                                  # fp32 kernel
    (2, dict(B=2, Hq=4, Hkv=4, L=(100, 900))),                   # key-split bf16 kernel, several chunks
    (4, dict(B=1, Hq=16, Hkv=2, L=(700, 700))),                  # row-split bf16 kernel (8 query heads per KV head)
])
@pytest.mark.parametrize("scale", [0.03, 0.25])
def test_softmax_scale_given_by_the_caller(cfg_id, kw, scale):
    """softmax_scale > 0 replaces the default 1/sqrt(D); both sides get the same value.  A flatter and a sharper
    softmax than the default (0.088 / 0.125) move the result well outside the tolerance if the scale is ignored."""
    from paper_2402_13720_amd import binding as ob
    from gpu_util import upload_attention
    cfg = W.scaled(W.CONFIGS[cfg_id], **kw)
    inp = W.make_attention_inputs(cfg, 900 + cfg_id)
    t = upload_attention(cfg, inp, False)
    lse = torch.full((cfg.B, cfg.Hq, cfg.T), float("nan"), dtype=torch.float32, device=DEV)
    out = ob.ouro_verify_attn(t["q"], t["k_cache"], t["v_cache"], t["cu_seqlens"], t["k_blk"], t["v_blk"], t["meta"],
                              max_seqlen=t["max_seqlen"], lse=lse, softmax_scale=scale)
    torch.cuda.synchronize()
    ref = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                             inp["pid"], inp["boff"], scale=scale)
    dflt = _oracle(inp)
    assert np.abs(to_np64(out) - ref["out"]).max() <= attn_tol(cfg)
    assert np.abs(to_np64(lse) - ref["lse"]).max() <= (1e-2 if cfg.dtype == "bf16" else 1e-5)
    assert np.abs(dflt["out"] - ref["out"]).max() > 5 * attn_tol(cfg)          # the case can tell the two scales apart


@pytest.mark.parametrize("B, rw, equal", [(2, 1, True), (16, 1, False), (63, 1, False), (64, 1, False), (64, 4, False),
                                          (65, 1, False), (70, 4, False), (40, 2, True), (130, 1, False),
                                          (256, 1, False), (256, 4, False), (257, 1, False)])
def test_bf16_many_sequences_taken_by_length_rank(B, rw, equal):
    """The bf16 kernels hand sequences to workgroups by length rank (every wave ranks the lengths itself: one per lane up
    to 64 sequences, four per lane up to 256; with more sequences, in batch order): every sequence must still be served
    exactly once, with lengths all different, with ties, at and around every one of those limits."""
    lens = np.full(B, 97) if equal else np.random.default_rng(B).permutation(B) * 5 % 211   # several ties, one empty
    cfg = W.scaled(W.CONFIGS[2], B=B, Hq=2, Hkv=2, L=(0, 300), gamma=4, K=2, beta_p=3)
    inp = W.make_attention_inputs(cfg, 99 + B, seqlens=lens)
    _check(cfg, inp, head_major=bool(B & 1), rw=rw)


@pytest.mark.parametrize("case", range(48))
def test_bf16_seeded_random_shapes(case):
    """A seeded sweep over shapes nobody picked by hand: batch (up to 70 sequences), head grouping (up to 8 query heads
    per KV head), draft layout, cache lengths from empty to a few dozen tiles, the kernel variant, the chunk length, the
    cache layout and the branch rule (including phrases that hang off the cached prefix, branch offset -1) all drawn per
    case."""
    rng = np.random.default_rng(7000 + case)
    Hkv = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([1, 1, 2, 4, 8]))
    gamma = int(rng.integers(1, 33))
    K = int(rng.integers(0, 9))
    bp = int(rng.integers(1, 7)) if K else 0
    while gamma + K * bp > 128:
        K -= 1
    lo = int(rng.choice([0, 1, 31, 64, 200, 900]))
    hi = lo + int(rng.choice([0, 1, 33, 250, 700, 2500]))
    B = int(rng.choice([1, 2, 3, 5, 9, 17, 33, 70]))
    cfg = W.scaled(W.CONFIGS[2], B=B, Hq=Hkv * G, Hkv=Hkv, L=(lo, hi), gamma=gamma, K=K, beta_p=bp)
    rw = int(rng.choice([0, 1, 2, 4, 4 + 0x80]))
    chunk = int(rng.choice([0, 128, 256, 384, 1024]))
    inp = W.make_attention_inputs(cfg, 8000 + case, branch=str(rng.choice(["uniform", "last", "any"])))
    _check(cfg, inp, head_major=bool(rng.integers(0, 2)), rw=rw, chunk=chunk)
