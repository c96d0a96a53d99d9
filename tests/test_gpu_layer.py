"""GPU parity of the layer pieces around the attention (positions + rotary embedding, RMSNorm, projections, SwiGLU)
against the layer oracle, and of one whole verifying layer chained on the GPU."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as LO, verify_oracle as O
from paper_2402_13720_amd import binding as ob, workloads as W
from gpu_util import DEV, to_np64

pytestmark = pytest.mark.gpu
BF16_EPS = 2.0 ** -8          # relative spacing bound of a value rounded to bf16 (RNE: error <= 2^-9 |x|)


def _bf(x):
    return W.round_to_bf16(np.asarray(x, dtype=np.float32))


def _up(x, dt=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(dt).contiguous()


@pytest.mark.parametrize("cfg_id, kw, dt", [
    (1, dict(B=3, L=(0, 200)), torch.float32),
    (2, dict(B=2, Hq=4, Hkv=2, L=(0, 300)), torch.bfloat16),             # grouped-query: fewer key/value heads
    (5, dict(B=4, Hq=4, Hkv=4, L=(512, 8192)), torch.bfloat16),
    (1, dict(B=2, Hq=3, Hkv=1, D=6, L=(0, 50)), torch.float32),          # head dim without 16-byte vectors
])
def test_rope_block_from_fused_projection(cfg_id, kw, dt):
    """Second form of ouro_rope_block: rows [q heads | k heads | v heads] of a fused projection in, q and k_blk rotated
    and v_blk copied out; against the oracle's rotation of the split operands, and bit for bit against the in-place form."""
    cfg = W.scaled(W.CONFIGS[cfg_id], **kw)
    inp = W.make_attention_inputs(cfg, 400 + cfg_id, branch="uniform")
    cu = inp["cu_seqlens"]
    lens = np.diff(cu).astype(np.int32)
    pos_ref = LO.block_positions(inp["pid"], inp["boff"], lens)
    q_ref, k_ref = LO.rope(inp["q"], pos_ref), LO.rope(inp["k_blk"], pos_ref)
    fused = np.concatenate([inp["q"], inp["k_blk"], inp["v_blk"]], axis=2).reshape(cfg.B * cfg.T, -1)
    qkv = _up(fused, dt)
    snapshot = qkv.clone()
    q = torch.full((cfg.B, cfg.T, cfg.Hq, cfg.D), 7.0, dtype=dt, device=DEV)
    k = torch.full((cfg.B, cfg.T, cfg.Hkv, cfg.D), 7.0, dtype=dt, device=DEV)
    v = torch.full((cfg.B, cfg.T, cfg.Hkv, cfg.D), 7.0, dtype=dt, device=DEV)
    meta, cu_d = ob.pack_meta(inp["pid"], inp["boff"]).to(DEV), torch.from_numpy(cu).to(DEV)
    pos = torch.empty(cfg.B, cfg.T, dtype=torch.int32, device=DEV)
    ob.ouro_rope_block(q, k, meta, cu_d, positions=pos, qkv=qkv, v_blk=v)
    q2, k2 = _up(inp["q"], dt), _up(inp["k_blk"], dt)
    ob.ouro_rope_block(q2, k2, meta, cu_d)
    torch.cuda.synchronize()
    assert np.array_equal(pos.cpu().numpy(), pos_ref)
    assert torch.equal(qkv, snapshot)                                    # the source is read only
    assert torch.equal(v, _up(inp["v_blk"], dt))                         # a copy: exact
    assert torch.equal(q, q2) and torch.equal(k, k2)                     # same arithmetic as the in-place form
    xmax = float(np.abs(inp["q"]).max())
    tol = 2.0 * xmax * (pos_ref.max() * 2.0 ** -23 + (BF16_EPS if dt == torch.bfloat16 else 2.0 ** -22))
    assert np.abs(to_np64(q) - q_ref).max() <= tol and np.abs(to_np64(k) - k_ref).max() <= tol


@pytest.mark.parametrize("cfg_id, kw, dt", [
    (1, dict(B=3, L=(0, 200)), torch.float32),
    (2, dict(B=2, Hq=4, Hkv=2, L=(0, 300)), torch.bfloat16),
    (5, dict(B=4, Hq=4, Hkv=4, L=(512, 8192)), torch.bfloat16),          # positions in the thousands
])
@pytest.mark.parametrize("with_len", [False, True])
def test_rope_block(cfg_id, kw, dt, with_len):
    cfg = W.scaled(W.CONFIGS[cfg_id], **kw)
    inp = W.make_attention_inputs(cfg, 300 + cfg_id, branch="uniform")
    inp["boff"][0, cfg.gamma:cfg.gamma + cfg.beta_p] = -1                # one phrase hangs off the prefix
    cu = inp["cu_seqlens"]
    lens = np.diff(cu).astype(np.int32)
    if with_len:                                                        # regions with room: lengths given apart
        lens = np.maximum(lens - 3, 0).astype(np.int32)
    pos_ref = LO.block_positions(inp["pid"], inp["boff"], lens)
    q_ref, k_ref = LO.rope(inp["q"], pos_ref), LO.rope(inp["k_blk"], pos_ref)
    q, k = _up(inp["q"], dt), _up(inp["k_blk"], dt)
    pos = torch.empty(cfg.B, cfg.T, dtype=torch.int32, device=DEV)
    ob.ouro_rope_block(q, k, ob.pack_meta(inp["pid"], inp["boff"]).to(DEV), torch.from_numpy(cu).to(DEV),
                       seq_len=torch.from_numpy(lens).to(DEV) if with_len else None, positions=pos)
    torch.cuda.synchronize()
    assert np.array_equal(pos.cpu().numpy(), pos_ref)                   # integer work: exact
    xmax = float(np.abs(inp["q"]).max())
    # fp32 angle = pos * inv_freq carries a relative 2^-23 error -> pos_max * 2^-23 radians; outputs then round to dt
    tol = 2.0 * xmax * (pos_ref.max() * 2.0 ** -23 + (BF16_EPS if dt == torch.bfloat16 else 2.0 ** -22))
    assert np.abs(to_np64(q) - q_ref).max() <= tol and np.abs(to_np64(k) - k_ref).max() <= tol


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("R, Hd", [(1, 64), (64, 4096), (37, 5120)])
def test_rmsnorm(dt, R, Hd):
    rng = np.random.default_rng(R + Hd)
    x, g = _bf(rng.standard_normal((R, Hd)) * 3.0), _bf(1.0 + 0.1 * rng.standard_normal(Hd))
    ref = LO.rmsnorm(x, g, 1e-5)
    out = ob.ouro_rmsnorm(_up(x, dt), _up(g, dt), 1e-5)
    torch.cuda.synchronize()
    tol = np.abs(ref).max() * (BF16_EPS if dt == torch.bfloat16 else 1e-5)
    assert np.abs(to_np64(out) - ref).max() <= tol


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_silu_mul(dt):
    rng = np.random.default_rng(9)
    gu = _bf(rng.standard_normal((33, 2 * 1000)) * 4.0)
    ref = LO.silu_mul(gu)
    out = ob.ouro_silu_mul(_up(gu, dt))
    torch.cuda.synchronize()
    tol = np.abs(ref).max() * (BF16_EPS if dt == torch.bfloat16 else 1e-5)
    assert np.abs(to_np64(out) - ref).max() <= tol


@pytest.mark.parametrize("R, K, N", [(64, 4096, 1024), (1, 64, 8), (37, 320, 264), (128, 1024, 640), (300, 512, 384)])
@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("with_res", [False, True])
def test_linear(R, K, N, tiled, with_res):
    rng = np.random.default_rng(R * 7 + N)
    x, w = _bf(rng.standard_normal((R, K))), _bf(rng.standard_normal((N, K)) * 0.05)
    res = _bf(rng.standard_normal((R, N))) if with_res else None
    ref = LO.linear(x, w, res)
    w_d = _up(w)
    if tiled:
        w_d = ob.ouro_lmhead_pack_w(w_d)
    out = ob.ouro_linear(_up(x), w_d, residual=None if res is None else _up(res))
    torch.cuda.synchronize()
    # fp32 accumulation of exact bf16 products (error ~1e-6 relative to the sum of magnitudes), one bf16 rounding
    tol = np.abs(ref).max() * BF16_EPS + 1e-4
    assert np.abs(to_np64(out) - ref).max() <= tol


@pytest.mark.parametrize("R,K,F,tiled,ksplit", [
    (64, 256, 344, True, 0),        # F not a multiple of 64: the last slab is ragged
    (128, 320, 64, False, 0),       # 128-row instance
    (70, 320, 136, True, 3),        # k range split: the activation is applied by the reduction kernel
    (1, 64, 8, False, 0),
])
def test_linear_swiglu_epilogue(R, K, F, tiled, ksplit):
    """Gate and up projection with the gate applied in the epilogue: interleaved (gate_j, up_j) weight rows in, [R, F] out,
    against the oracle's projection followed by its SiLU gate (no bf16 rounding of the pre-activations in between)."""
    rng = np.random.default_rng(R + K + F)
    x = _bf(rng.standard_normal((R, K)))
    wg, wu = _bf(rng.standard_normal((F, K)) * 0.08), _bf(rng.standard_normal((F, K)) * 0.08)
    ref = LO.silu_mul(np.concatenate([LO.linear(x, wg), LO.linear(x, wu)], axis=1))
    w_d = ob.ouro_interleave_gate_up(_up(wg), _up(wu))
    assert torch.equal(w_d[0::2], _up(wg)) and torch.equal(w_d[1::2], _up(wu))
    if tiled:
        w_d = ob.ouro_lmhead_pack_w(w_d)
    out = ob.ouro_linear(_up(x), w_d, swiglu=True, ksplit=ksplit)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (R, F)
    # fp32 product and gate, one bf16 rounding; the gate's slope is at most 1.1, so the product's error carries over
    tol = np.abs(ref).max() * BF16_EPS + 1e-4
    assert np.abs(to_np64(out) - ref).max() <= tol


@pytest.mark.parametrize("R,K,N,tiled,ksplit,with_res,swiglu", [
    (64, 320, 264, True, 0, False, False),
    (64, 4096, 256, True, 0, True, False),      # the heuristic splits the k range (2 slabs): row sums go through the reduction
    (128, 320, 136, False, 0, True, False),     # 128-row instance
    (70, 320, 272, True, 3, False, True),       # split k range, ragged rows, with the SwiGLU gate on top
    (33, 192, 48, False, 0, False, True),
    (1, 64, 8, False, 0, False, False),
])
def test_linear_with_rmsnorm_folded_in(R, K, N, tiled, ksplit, with_res, swiglu):
    """RMSNorm of the input inside the projection: rows of the product scaled by 1/sqrt(mean(x^2) + eps), the gain folded
    into the weight at load time.  Reference: the oracle's RMSNorm followed by its projection, with the folded weight
    the GPU gets (so that the comparison isolates the kernel), and separately the unfolded chain at a looser bound.
    The folded weight itself (a load-time library call) must equal the product rounded once to bf16, bit for bit."""
    rng = np.random.default_rng(R * 3 + K + N)
    eps = 1e-5
    x = _bf(rng.standard_normal((R, K)) * 1.7)
    w = _bf(rng.standard_normal((N, K)) * 0.05)
    g = _bf(1 + 0.2 * rng.standard_normal(K))
    res = _bf(rng.standard_normal((R, N))) if with_res else None
    w_fold_d = ob.ouro_fold_rmsnorm_gain(_up(w), _up(g))
    w_fold = w_fold_d.float().cpu().numpy().astype(np.float64)
    # the product of two bf16 values is exact in fp32 (8 + 8 significant bits), so one rounding defines the result
    assert np.array_equal(w_fold_d.float().cpu().numpy(), W.round_to_bf16(w.astype(np.float32) * g.astype(np.float32)[None, :]))
    ones = np.ones(K)
    pre = LO.linear(LO.rmsnorm(x, ones, eps), w_fold)                   # = rinv * (x . w_fold^T), fp64
    pre_unfolded = LO.linear(LO.rmsnorm(x, g, eps), w)
    post = (lambda y: LO.silu_mul(np.concatenate([y[:, 0::2], y[:, 1::2]], axis=1))) if swiglu else (lambda y: y)
    ref = post(pre) + (0 if res is None else res)
    ref_unfolded = post(pre_unfolded) + (0 if res is None else res)
    w_use = ob.ouro_lmhead_pack_w(w_fold_d) if tiled else w_fold_d
    out = ob.ouro_linear(_up(x), w_use, residual=None if res is None else _up(res), swiglu=swiglu, rms_eps=eps,
                         ksplit=ksplit)
    torch.cuda.synchronize()
    got = to_np64(out)
    tol = np.abs(ref).max() * BF16_EPS + 1e-4
    assert np.abs(got - ref).max() <= tol
    # folding rounds every weight once more (relative 2^-9 each, incoherent over K terms)
    assert np.abs(got - ref_unfolded).max() <= tol + 4 * BF16_EPS * np.abs(pre_unfolded).max()


@pytest.mark.parametrize("ksplit", [2, 3, 5])
def test_linear_uneven_k_split(ksplit):
    """The k range split over workgroups, including splits that do not divide the 5 k-tiles evenly (one share empty)."""
    rng = np.random.default_rng(ksplit)
    x, w, res = _bf(rng.standard_normal((70, 320))), _bf(rng.standard_normal((264, 320)) * 0.05), _bf(rng.standard_normal((70, 264)))
    ref = LO.linear(x, w, res)
    ws = torch.full((ksplit * 70 * (264 + 1) * 4,), 0xA5, dtype=torch.uint8, device=DEV)   # contents must not matter
    out = ob.ouro_linear(_up(x), _up(w), residual=_up(res), workspace=ws, ksplit=ksplit)
    torch.cuda.synchronize()
    assert np.abs(to_np64(out) - ref).max() <= np.abs(ref).max() * BF16_EPS + 1e-4


def test_one_verifying_layer_chained_on_the_gpu():
    """x -> RMSNorm -> fused QKV projection -> rotary embedding at the draft positions -> draft-block attention ->
    output projection + residual -> RMSNorm -> fused gate/up projection -> SwiGLU -> down projection + residual.
    The oracle chain rounds to bf16 wherever the GPU chain stores bf16, so both see the same intermediate values up
    to the rounding of each stage's own arithmetic."""
    cfg = W.scaled(W.CONFIGS[2], B=2, Hq=8, Hkv=4, L=(40, 700), gamma=8, K=4, beta_p=6)   # hidden 1024, T = 32
    Hd, D, F = cfg.Hq * cfg.D, cfg.D, 1536
    rng = np.random.default_rng(77)
    inp = W.make_attention_inputs(cfg, 4242)
    lens = np.diff(inp["cu_seqlens"]).astype(np.int32)
    R = cfg.B * cfg.T
    x = _bf(rng.standard_normal((R, Hd)))
    g1, g2 = _bf(1 + 0.1 * rng.standard_normal(Hd)), _bf(1 + 0.1 * rng.standard_normal(Hd))
    nqkv = (cfg.Hq + 2 * cfg.Hkv) * D
    wqkv, wo = _bf(rng.standard_normal((nqkv, Hd)) * Hd ** -0.5), _bf(rng.standard_normal((Hd, Hd)) * Hd ** -0.5)
    wgu, wd = _bf(rng.standard_normal((2 * F, Hd)) * Hd ** -0.5), _bf(rng.standard_normal((Hd, F)) * F ** -0.5)

    # ---- oracle chain (fp64 arithmetic, bf16 storage between the stages)
    h = _bf(LO.rmsnorm(x, g1, 1e-5))
    qkv = _bf(LO.linear(h, wqkv)).reshape(cfg.B, cfg.T, cfg.Hq + 2 * cfg.Hkv, D)
    q0, k0, v0 = qkv[:, :, :cfg.Hq], qkv[:, :, cfg.Hq:cfg.Hq + cfg.Hkv], qkv[:, :, cfg.Hq + cfg.Hkv:]
    pos = LO.block_positions(inp["pid"], inp["boff"], lens)
    q1, k1 = _bf(LO.rope(q0, pos)), _bf(LO.rope(k0, pos))
    att = _bf(O.verify_attention(q1, inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], k1, np.ascontiguousarray(v0),
                                 inp["pid"], inp["boff"])["out"]).reshape(R, Hd)
    x1 = _bf(LO.linear(att, wo, x))
    h2 = _bf(LO.rmsnorm(x1, g2, 1e-5))
    act = _bf(LO.silu_mul(_bf(LO.linear(h2, wgu))))
    ref = LO.linear(act, wd, x1)

    # ---- GPU chain
    meta = ob.pack_meta(inp["pid"], inp["boff"]).to(DEV)
    cu_d = torch.from_numpy(inp["cu_seqlens"]).to(DEV)
    x_d = _up(x)
    h_d = ob.ouro_rmsnorm(x_d, _up(g1), 1e-5)
    qkv_d = ob.ouro_linear(h_d, ob.ouro_lmhead_pack_w(_up(wqkv))).view(cfg.B, cfg.T, cfg.Hq + 2 * cfg.Hkv, D)
    q_d = qkv_d[:, :, :cfg.Hq].contiguous()
    k_d = qkv_d[:, :, cfg.Hq:cfg.Hq + cfg.Hkv].contiguous()
    v_d = qkv_d[:, :, cfg.Hq + cfg.Hkv:].contiguous()
    ob.ouro_rope_block(q_d, k_d, meta, cu_d)
    att_d = ob.ouro_verify_attn(q_d, _up(inp["k_cache"]), _up(inp["v_cache"]), cu_d, k_d, v_d, meta, int(lens.max()))
    x1_d = ob.ouro_linear(att_d.view(R, Hd), ob.ouro_lmhead_pack_w(_up(wo)), residual=x_d)
    h2_d = ob.ouro_rmsnorm(x1_d, _up(g2), 1e-5)
    act_d = ob.ouro_silu_mul(ob.ouro_linear(h2_d, ob.ouro_lmhead_pack_w(_up(wgu))))
    out_d = ob.ouro_linear(act_d, ob.ouro_lmhead_pack_w(_up(wd)), residual=x1_d)
    torch.cuda.synchronize()
    err = np.abs(to_np64(out_d) - ref).max()
    scale = np.abs(ref).max()
    print("layer chain: max-abs err %.3g on outputs of magnitude %.3g" % (err, scale), flush=True)
    # each of the ~8 bf16 stores can differ by one rounding step between the chains; they add up incoherently
    assert err <= 8 * BF16_EPS * scale

    # ---- the same layer with the fused forms: rotary + split straight from the fused projection's output, and the
    # SwiGLU gate in the epilogue of the gate/up projection (weights interleaved at load time)
    qkv2 = ob.ouro_linear(h_d, ob.ouro_lmhead_pack_w(_up(wqkv)))
    q2, k2, v2 = torch.empty_like(q_d), torch.empty_like(k_d), torch.empty_like(v_d)
    ob.ouro_rope_block(q2, k2, meta, cu_d, qkv=qkv2, v_blk=v2)
    att2 = ob.ouro_verify_attn(q2, _up(inp["k_cache"]), _up(inp["v_cache"]), cu_d, k2, v2, meta, int(lens.max()))
    x1b = ob.ouro_linear(att2.view(R, Hd), ob.ouro_lmhead_pack_w(_up(wo)), residual=x_d)
    h2b = ob.ouro_rmsnorm(x1b, _up(g2), 1e-5)
    w_pairs = ob.ouro_lmhead_pack_w(ob.ouro_interleave_gate_up(_up(wgu[:F]), _up(wgu[F:])))
    act2 = ob.ouro_linear(h2b, w_pairs, swiglu=True)
    out2 = ob.ouro_linear(act2, ob.ouro_lmhead_pack_w(_up(wd)), residual=x1b)
    torch.cuda.synchronize()
    assert torch.equal(q2, q_d) and torch.equal(k2, k_d) and torch.equal(v2, v_d) and torch.equal(x1b, x1_d)
    err2 = np.abs(to_np64(out2) - ref).max()
    print("layer chain, fused forms: max-abs err %.3g" % err2, flush=True)
    assert err2 <= 8 * BF16_EPS * scale

    # ---- and with both RMSNorms folded into the projections that follow them: 7 calls for the layer
    wqkv_f = ob.ouro_lmhead_pack_w(ob.ouro_fold_rmsnorm_gain(_up(wqkv), _up(g1)))
    wgu_f = ob.ouro_lmhead_pack_w(ob.ouro_fold_rmsnorm_gain(ob.ouro_interleave_gate_up(_up(wgu[:F]), _up(wgu[F:])), _up(g2)))
    qkv3 = ob.ouro_linear(x_d, wqkv_f, rms_eps=1e-5)
    q3, k3, v3 = torch.empty_like(q_d), torch.empty_like(k_d), torch.empty_like(v_d)
    ob.ouro_rope_block(q3, k3, meta, cu_d, qkv=qkv3, v_blk=v3)
    att3 = ob.ouro_verify_attn(q3, _up(inp["k_cache"]), _up(inp["v_cache"]), cu_d, k3, v3, meta, int(lens.max()))
    x1c = ob.ouro_linear(att3.view(R, Hd), ob.ouro_lmhead_pack_w(_up(wo)), residual=x_d)
    act3 = ob.ouro_linear(x1c, wgu_f, swiglu=True, rms_eps=1e-5)
    out3 = ob.ouro_linear(act3, ob.ouro_lmhead_pack_w(_up(wd)), residual=x1c)
    torch.cuda.synchronize()
    err3 = np.abs(to_np64(out3) - ref).max()
    print("layer chain, norms folded into the projections: max-abs err %.3g" % err3, flush=True)
    assert err3 <= 8 * BF16_EPS * scale


def test_rope_block_with_a_given_base():
    """base > 0 replaces the default 10000 (a long-context model's 500000 here); the two differ far beyond the tolerance."""
    cfg = W.scaled(W.CONFIGS[2], B=2, Hq=4, Hkv=2, L=(3000, 5000))
    inp = W.make_attention_inputs(cfg, 555)
    lens = np.diff(inp["cu_seqlens"]).astype(np.int32)
    pos_ref = LO.block_positions(inp["pid"], inp["boff"], lens)
    q_ref, q_dflt = LO.rope(inp["q"], pos_ref, base=500000.0), LO.rope(inp["q"], pos_ref)
    k_ref = LO.rope(inp["k_blk"], pos_ref, base=500000.0)
    q, k = _up(inp["q"]), _up(inp["k_blk"])
    ob.ouro_rope_block(q, k, ob.pack_meta(inp["pid"], inp["boff"]).to(DEV), torch.from_numpy(inp["cu_seqlens"]).to(DEV),
                       base=500000.0)
    torch.cuda.synchronize()
    xmax = float(np.abs(inp["q"]).max())
    tol = 2.0 * xmax * (pos_ref.max() * 2.0 ** -23 + BF16_EPS)
    assert np.abs(to_np64(q) - q_ref).max() <= tol and np.abs(to_np64(k) - k_ref).max() <= tol
    assert np.abs(q_dflt - q_ref).max() > 20 * tol


def test_layer_ops_edge_shapes():
    """One-token blocks, a single row, odd sizes that take the scalar paths, in-place RMSNorm."""
    rng = np.random.default_rng(31)
    cfg = W.scaled(W.CONFIGS[2], B=3, Hq=2, Hkv=1, L=(0, 50), gamma=1, K=0, beta_p=0, D=128)     # T = 1
    inp = W.make_attention_inputs(cfg, 88)
    lens = np.diff(inp["cu_seqlens"]).astype(np.int32)
    pos_ref = LO.block_positions(inp["pid"], inp["boff"], lens)
    q, k = _up(inp["q"]), _up(inp["k_blk"])
    pos = torch.empty(cfg.B, 1, dtype=torch.int32, device=DEV)
    ob.ouro_rope_block(q, k, ob.pack_meta(inp["pid"], inp["boff"]).to(DEV), torch.from_numpy(inp["cu_seqlens"]).to(DEV),
                       positions=pos)
    torch.cuda.synchronize()
    assert np.array_equal(pos.cpu().numpy(), pos_ref) and np.array_equal(pos_ref[:, 0], lens)
    assert np.abs(to_np64(q) - LO.rope(inp["q"], pos_ref)).max() <= 2 * np.abs(inp["q"]).max() * BF16_EPS
    # head dim 12 (not a multiple of 16): scalar rotary path, fp32
    x = rng.standard_normal((1, 1, 3, 12)).astype(np.float32)
    xk = rng.standard_normal((1, 1, 1, 12)).astype(np.float32)
    qd, kd = _up(x, torch.float32), _up(xk, torch.float32)
    ob.ouro_rope_block(qd, kd, ob.pack_meta(np.zeros((1, 1), np.int16), np.zeros((1, 1), np.int16)).to(DEV),
                       torch.tensor([0, 9], dtype=torch.int64, device=DEV))
    torch.cuda.synchronize()
    assert np.abs(to_np64(qd) - LO.rope(x, np.array([[9]]))).max() <= 1e-5
    # RMSNorm: a row length that is not a multiple of 8, a long row (beyond the register-resident path), in place
    for Hd in (100, 20000):
        xr, g = _bf(rng.standard_normal((3, Hd))), _bf(1 + 0.1 * rng.standard_normal(Hd))
        xd = _up(xr)
        ob.ouro_rmsnorm(xd, _up(g), 1e-6, out=xd)
        torch.cuda.synchronize()
        ref = LO.rmsnorm(xr, g, 1e-6)
        assert np.abs(to_np64(xd) - ref).max() <= np.abs(ref).max() * BF16_EPS


@pytest.mark.parametrize("case", range(16))
def test_linear_seeded_random_options(case):
    """A seeded sweep over ouro_linear's options together: rows on both sides of the 64-row instance boundary, ragged last
    slabs, k splits that the heuristic would not pick, residual, the SwiGLU epilogue and the folded RMSNorm."""
    rng = np.random.default_rng(600 + case)
    R = int(rng.choice([1, 17, 64, 65, 128, 130]))
    K = 64 * int(rng.integers(1, 8))
    swiglu = bool(rng.integers(0, 2))
    N = 16 * int(rng.integers(1, 30)) if swiglu else 8 * int(rng.integers(1, 60))
    rms = bool(rng.integers(0, 2))
    with_res = (not swiglu) and bool(rng.integers(0, 2))
    ksplit = int(rng.choice([0, 0, 2, 3]))
    eps = 1e-5
    x = _bf(rng.standard_normal((R, K)) * 1.3)
    w = _bf(rng.standard_normal((N, K)) * 0.06)
    res = _bf(rng.standard_normal((R, N))) if with_res else None
    pre = LO.linear(LO.rmsnorm(x, np.ones(K), eps), w) if rms else LO.linear(x, w)
    ref = LO.silu_mul(np.concatenate([pre[:, 0::2], pre[:, 1::2]], axis=1)) if swiglu else pre
    if res is not None:
        ref = ref + res
    w_d = _up(w)
    if rng.integers(0, 2):
        w_d = ob.ouro_lmhead_pack_w(w_d)
    out = ob.ouro_linear(_up(x), w_d, residual=None if res is None else _up(res), swiglu=swiglu, rms_eps=eps if rms else 0.0,
                         ksplit=ksplit)
    torch.cuda.synchronize()
    assert np.abs(to_np64(out) - ref).max() <= np.abs(ref).max() * BF16_EPS + 1e-4
