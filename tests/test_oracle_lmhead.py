"""Pins for the oracle's LM head + greedy pick (no GPU)."""
import numpy as np
import torch

from oracle import verify_oracle as O


def test_hand_example():
    # logits = h W^T with W stored [V, Hd]: rows of W are token embeddings.
    h = np.array([[1.0, 2.0], [3.0, -1.0]])
    w = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, -1.0]])
    # row 0: [1, 2, 3, -3] -> token 2, margin 1 ; row 1: [3, -1, 2, -2] -> token 0, margin 1
    r = O.lmhead_argmax(h, w)
    assert r["argmax"].tolist() == [2, 0]
    np.testing.assert_allclose(r["top1"], [3.0, 3.0])
    np.testing.assert_allclose(r["top2"], [2.0, 2.0])
    np.testing.assert_allclose(r["margin"], [1.0, 1.0])


def test_matches_library_matmul():
    rng = np.random.default_rng(0)
    h, w = rng.standard_normal((9, 33)), rng.standard_normal((57, 33)) * 0.02
    r = O.lmhead_argmax(h, w)
    logits = (torch.from_numpy(h) @ torch.from_numpy(w).T).numpy()
    assert np.array_equal(r["argmax"], logits.argmax(1))
    np.testing.assert_allclose(r["top1"], logits.max(1), atol=1e-14)
    srt = np.sort(logits, axis=1)
    np.testing.assert_allclose(r["margin"], srt[:, -1] - srt[:, -2], atol=1e-14)


def test_planted_winner():
    """Row v* of W set to c*h_r makes token v* win row r whenever c*|h_r|^2 exceeds every other logit."""
    rng = np.random.default_rng(1)
    h = rng.standard_normal((6, 40))
    w = rng.standard_normal((100, 40)) * 0.02
    plant = [17, 3, 99, 0, 50, 51]
    for r, v in enumerate(plant):
        w[v] = 10.0 * h[r]
    res = O.lmhead_argmax(h, w)
    assert res["argmax"].tolist() == plant
    np.testing.assert_allclose(res["top1"], 10.0 * (h * h).sum(1), rtol=1e-13)


def test_ties_go_to_lowest_token_id():
    h = np.array([[1.0, 1.0]])
    w = np.zeros((8, 2))
    w[5] = w[2] = w[7] = [2.0, 3.0]
    r = O.lmhead_argmax(h, w)
    assert r["argmax"].tolist() == [2]
    assert r["margin"][0] == 0.0
