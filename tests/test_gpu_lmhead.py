"""GPU parity: ouro_lmhead_argmax against the fp64 oracle.  Arg-max ids must be bit-exact except on rows
whose oracle top-2 margin is below 1e-3 (reported)."""
import functools

import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import binding as ob, workloads as W
from gpu_util import DEV, torch_dtype

pytestmark = pytest.mark.gpu

MARGIN = 1e-3


def _run(cfg, hidden, w, tiled=False):
    dt = torch_dtype(cfg)
    h_d = torch.from_numpy(hidden).to(DEV).to(dt).contiguous()
    w_d = torch.from_numpy(w).to(DEV).to(dt).contiguous()
    if tiled:
        w_d = ob.ouro_lmhead_pack_w(w_d)
    mx = torch.empty(hidden.shape[0], dtype=torch.float32, device=DEV)
    arg = ob.ouro_lmhead_argmax(h_d, w_d, max_out=mx)
    torch.cuda.synchronize()
    return arg.cpu().numpy(), mx.cpu().numpy()


def _check(cfg, hidden, w, rows=None, tiled=False, ref=None):
    arg, mx = _run(cfg, hidden, w, tiled)
    sel = np.arange(hidden.shape[0]) if rows is None else np.asarray(rows)
    if ref is None:
        ref = O.lmhead_argmax(hidden[sel], w)
    bad = [(int(r), int(arg[r]), int(ref["argmax"][i]), float(ref["margin"][i]))
           for i, r in enumerate(sel) if arg[r] != ref["argmax"][i]]
    print("%s: R=%d V=%d Hd=%d  exact on %d/%d checked rows; exempt (margin<%.0e): %s"
          % (cfg.name, hidden.shape[0], w.shape[0], w.shape[1], len(sel) - len(bad), len(sel), MARGIN, bad), flush=True)
    assert all(m < MARGIN for *_, m in bad), bad
    tol = 2e-3 if cfg.dtype == "bf16" else 2e-5
    assert np.abs(mx[sel] - ref["top1"]).max() <= tol * max(1.0, np.abs(ref["top1"]).max())
    assert (arg >= 0).all() and (arg < w.shape[0]).all()
    return arg


def test_config1_fp32():
    cfg = W.CONFIGS[1]
    for trial in range(3):
        s = W.seed_for(1, trial)
        _check(cfg, W.make_hidden(cfg, s), W.make_lmhead_weight(cfg, s))


@pytest.mark.parametrize("R,Hd,V", [(1, 64, 1), (5, 256, 300), (64, 512, 1000), (37, 1024, 129), (100, 256, 777),
                                    (128, 320, 1025), (200, 192, 500), (512, 128, 260)])
@pytest.mark.parametrize("tiled", [False, True])
def test_bf16_shapes(R, Hd, V, tiled):
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=Hd // 64, Hkv=Hd // 64, D=64, V=V)
    assert cfg.hidden == Hd
    _check(cfg, W.make_hidden(cfg, 3, rows=R), W.make_lmhead_weight(cfg, 3), tiled=tiled)


@pytest.mark.parametrize("V,Hd", [(1, 64), (128, 64), (129, 192), (1000, 256), (32000, 4096)])
def test_pack_w_is_the_documented_reblocking(V, Hd):
    """[V, Hd] -> [ceil(V/128)][Hd/64][128][64], rows past V zero: a pure index permutation, bit-exact."""
    rng = np.random.default_rng(V)
    w = torch.from_numpy(rng.integers(-30000, 30000, size=(V, Hd)).astype(np.int16)).to(DEV).view(torch.bfloat16)
    packed = ob.ouro_lmhead_pack_w(w)
    torch.cuda.synchronize()
    got = packed.data.view(torch.int16).cpu().numpy()
    ns = (V + 127) // 128
    pad = np.zeros((ns * 128, Hd), np.int16)
    pad[:V] = w.view(torch.int16).cpu().numpy()
    want = pad.reshape(ns, 128, Hd // 64, 64).transpose(0, 2, 1, 3).reshape(-1)
    assert got.shape == want.shape and np.array_equal(got, want)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ties_go_to_lowest_id_within_and_across_slabs(dtype):
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=4, Hkv=4, D=64, V=1000, dtype=dtype)
    hidden = W.make_hidden(cfg, 4, rows=40)
    w = W.make_lmhead_weight(cfg, 4)
    big = W.round_to_bf16(np.random.default_rng(0).standard_normal(cfg.hidden).astype(np.float32))
    for v in (999, 700, 131, 130, 5):                      # identical rows: identical logits in any arithmetic
        w[v] = big
    hidden[:] = 0
    hidden[:, :] = big * np.float32(0.5)                   # every row prefers the planted embedding
    arg, _ = _run(cfg, hidden, w)
    assert (arg == 5).all()
    w[5] = 0
    arg, _ = _run(cfg, hidden, w)
    assert (arg == 130).all()
    w[130] = 0
    arg, _ = _run(cfg, hidden, w)
    assert (arg == 131).all()


def test_planted_winners_bf16():
    cfg = W.scaled(W.CONFIGS[2], V=4000)
    hidden = W.make_hidden(cfg, 9)
    w = W.make_lmhead_weight(cfg, 9)
    rng = np.random.default_rng(1)
    plant = rng.choice(cfg.V, size=cfg.R, replace=False)
    for r, v in enumerate(plant):
        w[v] = hidden[r] * np.float32(0.25)                # exact in bf16 (power-of-two scale)
    arg, _ = _run(cfg, hidden, w)
    assert np.array_equal(arg, plant)


@functools.lru_cache(maxsize=1)
def _full_size_case(cfg_id):
    """(hidden, weight, oracle result on every row) of a workload at full size, shared by the two weight layouts."""
    cfg = W.CONFIGS[cfg_id]
    s = W.seed_for(cfg_id)
    hidden, w = W.make_hidden(cfg, s), W.make_lmhead_weight(cfg, s)
    return hidden, w, O.lmhead_argmax(hidden, w)


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("cfg_id", [2, 3, 4, 5])
def test_full_size_configs_every_row(cfg_id, tiled):
    cfg = W.CONFIGS[cfg_id]
    hidden, w, ref = _full_size_case(cfg_id)
    _check(cfg, hidden, w, tiled=tiled, ref=ref)


def test_workspace_is_reusable_across_shapes_and_calls():
    ws = torch.full((8 << 20,), 0xA5, dtype=torch.uint8, device=DEV)
    for (R, Hd, V, seed) in [(64, 512, 3000, 1), (200, 256, 1500, 2), (64, 512, 3000, 1)]:
        cfg = W.scaled(W.CONFIGS[2], B=1, Hq=Hd // 64, Hkv=Hd // 64, D=64, V=V)
        hidden, w = W.make_hidden(cfg, seed, rows=R), W.make_lmhead_weight(cfg, seed)
        ref = O.lmhead_argmax(hidden, w)
        h_d = torch.from_numpy(hidden).to(DEV).to(torch.bfloat16)
        w_d = torch.from_numpy(w).to(DEV).to(torch.bfloat16)
        assert ob.ouro_lmhead_argmax_workspace(h_d, w_d) <= ws.numel()
        for _ in range(2):
            arg = ob.ouro_lmhead_argmax(h_d, w_d, workspace=ws).cpu().numpy()
            bad = [r for r in range(R) if arg[r] != ref["argmax"][r] and ref["margin"][r] >= MARGIN]
            assert not bad


@pytest.mark.parametrize("case", range(20))
def test_bf16_seeded_random_shapes(case):
    """A seeded sweep over shapes nobody picked by hand: row counts on both sides of the 64 / 128 / 256 boundaries that
    select the kernel and its tiles, hidden sizes from one k-tile up, vocabularies with ragged last slabs, either layout."""
    rng = np.random.default_rng(9000 + case)
    R = int(rng.choice([1, 2, 31, 63, 64, 65, 100, 127, 128, 129, 200, 255, 256, 257, 300, 513]))
    Hd = 64 * int(rng.integers(1, 9))
    V = int(rng.choice([1, 7, 127, 128, 129, 255, 256, 257, 700, 1537]))
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=Hd // 64, Hkv=Hd // 64, D=64, V=V)
    _check(cfg, W.make_hidden(cfg, 50 + case, rows=R), W.make_lmhead_weight(cfg, 50 + case), tiled=bool(rng.integers(0, 2)))
