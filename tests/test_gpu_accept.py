"""GPU parity: ouro_accept against the oracle, bit-exact on every output."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import binding as ob, workloads as W
from golden_io import load_traces, meta_from_layout
from gpu_util import DEV

pytestmark = pytest.mark.gpu
KEYS = ("n_accept", "path", "bonus", "accept_idx", "main_A", "phrase_A", "n_match")


def _gpu(tok, argmax, pid, boff, root, gamma, K, bp):
    meta = ob.pack_meta(pid, boff).to(DEV)
    got = ob.ouro_accept(torch.from_numpy(tok.astype(np.int32)).to(DEV), torch.from_numpy(argmax.astype(np.int32)).to(DEV),
                         meta, None if root is None else torch.from_numpy(root.astype(np.int32)).to(DEV), gamma, K, bp)
    torch.cuda.synchronize()
    return {k: got[k].cpu().numpy() for k in KEYS}


def _compare(tok, argmax, pid, boff, root, gamma, K, bp):
    ref = O.accept(tok, argmax, pid, boff, root, gamma, K, bp)
    got = _gpu(tok, argmax, pid, boff, root, gamma, K, bp)
    for k in KEYS:
        assert np.array_equal(got[k], ref[k]), (k, got[k], ref[k])
    return ref


def test_handworked_traces():
    for t in load_traces("accept_traces.txt"):
        pid, boff = meta_from_layout(t["gamma"], t["K"], t["beta_p"], t["branch"])
        root = None if t["root"] is None else np.array([t["root"]])
        got = _gpu(t["tok"][None], t["argmax"][None], pid[None], boff[None], root, t["gamma"], t["K"], t["beta_p"])
        assert got["n_accept"][0] == t["n_accept"] and got["path"][0] == t["path"] and got["bonus"][0] == t["bonus"]
        assert got["accept_idx"][0].tolist() == t["idx"].tolist()
        assert got["main_A"][0] == t["A"] and got["phrase_A"][0].tolist() == t["Ahat"].tolist()


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("p_correct", [0.5, 0.9, 1.0, 0.0])
def test_config_shapes_random_drafts(cfg_id, p_correct):
    cfg = W.scaled(W.CONFIGS[cfg_id], B=max(W.CONFIGS[cfg_id].B, 7))
    rng = np.random.default_rng(cfg_id * 10 + int(p_correct * 10))
    for branch in ("uniform", "last"):
        pid, boff = W.make_block_meta(cfg, rng, branch)
        argmax = rng.integers(0, cfg.V, size=(cfg.B, cfg.T)).astype(np.int32)
        root = rng.integers(0, cfg.V, size=cfg.B).astype(np.int32)
        exp = np.stack([O.expected_tokens(argmax[b], pid[b], boff[b], int(root[b])) for b in range(cfg.B)])
        wrong = rng.integers(0, cfg.V, size=exp.shape)
        tok = np.where(rng.random(exp.shape) < p_correct, exp, wrong).astype(np.int32)
        ref = _compare(tok, argmax, pid, boff, root, cfg.gamma, cfg.K, cfg.beta_p)
        if p_correct == 1.0:
            assert (ref["n_accept"] >= cfg.gamma).all()
        _compare(tok, argmax, pid, boff, None, cfg.gamma, cfg.K, cfg.beta_p)


def test_edge_layouts():
    rng = np.random.default_rng(0)
    for gamma, K, bp in [(1, 0, 0), (128, 0, 0), (1, 63, 2), (2, 63, 2), (64, 1, 64), (5, 3, 1)]:
        T = gamma + K * bp
        for _ in range(4):
            branch = [int(rng.integers(-1, gamma)) for _ in range(K)]
            pid, boff = meta_from_layout(gamma, K, bp, branch)
            argmax = rng.integers(0, 6, size=(3, T)).astype(np.int32)
            tok = rng.integers(0, 6, size=(3, T)).astype(np.int32)
            root = rng.integers(0, 6, size=3).astype(np.int32)
            pid3, boff3 = np.repeat(pid[None], 3, 0), np.repeat(boff[None], 3, 0)
            _compare(tok, argmax, pid3, boff3, root, gamma, K, bp)
            _compare(tok, argmax, pid3, boff3, None, gamma, K, bp)
