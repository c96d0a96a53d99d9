"""Pins of the layer oracle (positions of block tokens, rotary embedding, RMSNorm, projections, SwiGLU)."""
import numpy as np
import pytest
import torch

from golden_io import meta_from_layout
from oracle import layer_oracle as LO, verify_oracle as O
from paper_2402_13720_amd import workloads as W


def test_positions_hand_example():
    # gamma = 4 main tokens, phrase 1 (3 tokens) off main index 1, phrase 2 (3 tokens) off the prefix, L = 10.
    # main: 10 11 12 13 ; phrase 1 follows main 0,1 -> 12 13 14 ; phrase 2 follows the prefix -> 10 11 12
    pid, boff = meta_from_layout(4, 2, 3, [1, -1])
    pos = LO.block_positions(pid[None], boff[None], np.array([10]))
    assert pos[0].tolist() == [10, 11, 12, 13, 12, 13, 14, 10, 11, 12]


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 5])
def test_positions_are_indices_in_the_linearised_drafts(cfg_id):
    """Lay each lengthened draft out as a linear sequence [prefix, main 0..b_j, phrase j] (Eq. (7)); a block
    token's position is its index there.  Also: depth = size of the conditioning set inside the block minus one."""
    cfg = W.CONFIGS[cfg_id]
    rng = np.random.default_rng(cfg_id)
    pid, boff = W.make_block_meta(W.scaled(cfg, B=2), rng)
    lens = np.array([17, 0])
    pos = LO.block_positions(pid, boff, lens)
    for b in range(2):
        assert pos[b, :cfg.gamma].tolist() == list(range(lens[b], lens[b] + cfg.gamma))
        for j in range(1, cfg.K + 1):
            lo = cfg.gamma + (j - 1) * cfg.beta_p
            bj = int(boff[b, lo])
            seq = list(range(bj + 1)) + list(range(lo, lo + cfg.beta_p))       # block indices of draft j, in order
            for idx_in_seq, t in enumerate(seq):
                assert pos[b, t] == lens[b] + idx_in_seq
        vis = O.block_visibility(pid[b], boff[b])
        assert np.array_equal(pos[b] - lens[b], vis.sum(axis=1) - 1)


def test_rope_equals_complex_multiplication_and_keeps_norms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 5, 3, 16))
    pos = rng.integers(0, 5000, size=(2, 5))
    y = LO.rope(x, pos, 10000.0)
    z = (x[..., :8] + 1j * x[..., 8:]) * np.exp(1j * pos[:, :, None, None] * 10000.0 ** (-np.arange(8) / 8.0))
    assert np.allclose(y[..., :8], z.real, atol=1e-12) and np.allclose(y[..., 8:], z.imag, atol=1e-12)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    assert np.array_equal(LO.rope(x, np.zeros((2, 5), dtype=int)), x)              # position 0 is the identity


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 1, 1, 32))
    k = rng.standard_normal((1, 1, 1, 32))
    s = [float((LO.rope(q, np.array([[m]])) * LO.rope(k, np.array([[m - 7]]))).sum()) for m in (7, 100, 4096)]
    assert np.allclose(s, s[0], atol=1e-9)


def test_rmsnorm_closed_forms():
    g = np.array([1.0, 2.0, 3.0, 4.0])
    assert np.allclose(LO.rmsnorm(np.full((1, 4), 5.0), g, 0.0), g)                 # constant row -> the gain
    x = np.array([[3.0, 4.0, 0.0, 0.0]])                                           # mean square = 25/4
    assert np.allclose(LO.rmsnorm(x, np.ones(4), 0.0), x / 2.5)
    assert np.allclose(LO.rmsnorm(x, np.ones(4), 0.75), x / np.sqrt(7.0))           # eps inside the root
    y = LO.rmsnorm(7.0 * x, g, 0.0)
    assert np.allclose(y, LO.rmsnorm(x, g, 0.0))                                    # scale invariance without eps


def test_linear_against_library_matmul():
    rng = np.random.default_rng(2)
    x, w, r = rng.standard_normal((5, 24)), rng.standard_normal((9, 24)), rng.standard_normal((5, 9))
    assert np.allclose(LO.linear(x, w), x @ w.T, atol=1e-12)
    want = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w)).numpy() + r
    assert np.allclose(LO.linear(x, w, r), want, atol=1e-12)
    assert LO.linear(x, w).shape == (5, 9)                                          # [rows, out features]


def test_silu_mul_closed_forms():
    gu = np.array([[0.0, 1.0, -1.0, 30.0, 2.0, 3.0, 4.0, 5.0]])
    y = LO.silu_mul(gu)[0]
    assert y[0] == 0.0
    assert np.isclose(y[1], 3.0 / (1.0 + np.exp(-1.0)))                             # silu(1) = 0.7310585786...
    assert np.isclose(y[2], -4.0 * (1.0 - 1.0 / (1.0 + np.exp(-1.0))))              # silu(-1) = -(1 - sigmoid(1))
    assert np.isclose(y[3], 150.0)                                                  # silu(z) -> z for large z
    want = (torch.nn.functional.silu(torch.from_numpy(gu[:, :4])) * torch.from_numpy(gu[:, 4:])).numpy()
    assert np.allclose(LO.silu_mul(gu), want, atol=1e-12)
