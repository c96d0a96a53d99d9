"""Pins for the oracle's acceptance rule (no GPU)."""
import itertools

import numpy as np
import pytest

from oracle import verify_oracle as O
from golden_io import load_traces, meta_from_layout

TRACES = load_traces("accept_traces.txt")


@pytest.mark.parametrize("i", range(len(TRACES)))
def test_handworked_traces(i):
    t = TRACES[i]
    pid, boff = meta_from_layout(t["gamma"], t["K"], t["beta_p"], t["branch"])
    r = O.accept_one(t["tok"], t["argmax"], pid, boff, t["root"], t["gamma"], t["K"], t["beta_p"])
    assert r["main_A"] == t["A"]
    assert r["phrase_A"].tolist() == t["Ahat"].tolist()
    assert r["path"] == t["path"]
    assert r["n_accept"] == t["n_accept"]
    assert r["bonus"] == t["bonus"]
    assert r["accept_idx"].tolist() == t["idx"].tolist()


def _lengthened_drafts(gamma, K, bp, branch):
    """Eq. (7) as explicit index lists: the main draft, and [main 0..b_j] + phrase j for each j."""
    lists = [list(range(gamma))]
    for j in range(1, K + 1):
        lo = gamma + (j - 1) * bp
        lists.append(list(range(branch[j - 1] + 1)) + list(range(lo, lo + bp)))
    return lists


def _enumerate_reference(tok, argmax, root, gamma, K, bp, branch):
    """Verify each lengthened draft one by one as an ordinary linear draft (Eq. (3) applied to each),
    keep the longest (lowest id on ties).  No eligibility logic: a phrase draft that fails inside the
    main part simply has the main draft's length or less."""
    best = (-1, None, None)
    for pidx, lst in enumerate(_lengthened_drafts(gamma, K, bp, branch)):
        n, prev = 0, None
        for t in lst:
            want = root if prev is None else argmax[prev]
            if want is not None and tok[t] != want:
                break
            n, prev = n + 1, t
        bonus = (root if root is not None else -1) if prev is None else argmax[prev]
        if n > best[0]:
            best = (n, lst[:n], bonus, pidx)
    return best


@pytest.mark.parametrize("gamma,K,bp", [(1, 1, 1), (2, 2, 2), (3, 2, 2), (3, 1, 2), (2, 2, 1)])
def test_exhaustive_match_patterns_against_one_by_one_enumeration(gamma, K, bp):
    T = gamma + K * bp
    rng = np.random.default_rng(gamma * 100 + K * 10 + bp)
    for branch in itertools.product(range(-1, gamma), repeat=K):
        pid, boff = meta_from_layout(gamma, K, bp, list(branch))
        argmax = rng.integers(10, 20, size=T)
        root = int(rng.integers(10, 20))
        for pattern in itertools.product([0, 1], repeat=T):
            want_tok = O.expected_tokens(argmax, pid, boff, root)   # only used to realise the pattern
            tok = np.where(np.array(pattern, bool), want_tok, 99)
            got = O.accept_one(tok, argmax, pid, boff, root, gamma, K, bp)
            n, idx, bonus, _ = _enumerate_reference(tok, argmax, root, gamma, K, bp, list(branch))
            assert got["n_accept"] == n
            assert got["accept_idx"][:n].tolist() == idx or \
                [tok[i] for i in got["accept_idx"][:n]] == [tok[i] for i in idx]
            assert (got["accept_idx"][n:] == -1).all()
            # bonus: when paths tie the bonus row differs only between rows predicting after equal contexts;
            # with random argmax per row it is only comparable when the accepted index lists coincide.
            if got["accept_idx"][:n].tolist() == idx:
                assert got["bonus"] == bonus


def test_expected_tokens_realises_parent_predictions():
    # independent of parents(): hand layout gamma=3, phrase1 off main 0, phrase2 off main 2
    pid, boff = meta_from_layout(3, 2, 2, [0, 2])
    a = np.array([10, 11, 12, 13, 14, 15, 16])
    assert O.expected_tokens(a, pid, boff, 7).tolist() == [7, 10, 11, 10, 13, 12, 15]
    assert O.parents(pid, boff).tolist() == [-1, 0, 1, 0, 3, 2, 5]


def test_all_correct_draft_is_fully_accepted():
    gamma, K, bp = 8, 4, 6
    pid, boff = meta_from_layout(gamma, K, bp, [3, 7, 7, 0])
    T = gamma + K * bp
    argmax = np.arange(100, 100 + T)
    tok = O.expected_tokens(argmax, pid, boff, 55)
    r = O.accept_one(tok, argmax, pid, boff, 55, gamma, K, bp)
    assert r["main_A"] == gamma and r["phrase_A"].tolist() == [bp] * K
    assert r["n_accept"] == gamma + bp and r["path"] == 2          # first phrase hanging off the last token
    assert r["bonus"] == argmax[gamma + 2 * bp - 1]
    assert r["n_match"] == gamma


def test_all_wrong_draft_accepts_nothing():
    gamma, K, bp = 4, 2, 3
    pid, boff = meta_from_layout(gamma, K, bp, [3, 3])
    argmax = np.arange(10)
    tok = np.full(10, 77)
    r = O.accept_one(tok, argmax, pid, boff, 5, gamma, K, bp)
    assert r["n_accept"] == 0 and r["path"] == 0 and r["bonus"] == 5 and (r["accept_idx"] == -1).all()
    r = O.accept_one(tok, argmax, pid, boff, None, gamma, K, bp)     # main 0 pre-accepted
    assert r["n_accept"] == 1 and r["bonus"] == argmax[0] and r["accept_idx"][0] == 0


def _toy_next(context):
    """A deterministic toy target model: next token is a hash of the whole context."""
    x = 1469598103934665603
    for t in context:
        x = ((x ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return int(x % 13)        # small vocabulary so that wrong drafts sometimes match by luck


@pytest.mark.parametrize("seed", range(40))
def test_lossless_replay_with_toy_target(seed):
    """Eq. (4): accepted tokens followed by the bonus are exactly what the target would generate
    token by token from the prefix; and no lengthened draft would have yielded more."""
    rng = np.random.default_rng(seed)
    gamma, K, bp = int(rng.integers(1, 7)), int(rng.integers(0, 4)), int(rng.integers(1, 5))
    branch = [int(rng.integers(-1, gamma)) for _ in range(K)]
    pid, boff = meta_from_layout(gamma, K, bp, branch)
    T = gamma + K * bp
    prefix = [int(x) for x in rng.integers(0, 13, size=4)]
    rollout = list(prefix)
    for _ in range(T + 2):
        rollout.append(_toy_next(rollout))
    truth = rollout[len(prefix):]
    # drafts: follow the truth with probability 0.8 per token along each lengthened draft
    tok = np.zeros(T, dtype=np.int64)
    lists = _lengthened_drafts(gamma, K, bp, branch)
    for lst in lists:
        for depth, t in enumerate(lst):
            if lst is lists[0] or t >= gamma:
                tok[t] = truth[depth] if rng.random() < 0.8 else int(rng.integers(0, 13))
    # target predictions for every block row: next(prefix + path to the row)
    argmax = np.zeros(T, dtype=np.int64)
    for lst in lists:
        for depth, t in enumerate(lst):
            argmax[t] = _toy_next(prefix + [int(tok[u]) for u in lst[:depth + 1]])
    root = _toy_next(prefix)
    r = O.accept_one(tok, argmax, pid, boff, root, gamma, K, bp)
    n = r["n_accept"]
    emitted = [int(tok[i]) for i in r["accept_idx"][:n]] + [r["bonus"]]
    assert emitted == truth[:n + 1]
    longest = max(next((d for d, t in enumerate(lst) if tok[t] != truth[d]), len(lst)) for lst in lists)
    assert n == longest


def test_batch_wrapper_and_match_count():
    gamma, K, bp = 4, 1, 2
    pid, boff = meta_from_layout(gamma, K, bp, [3])
    argmax = np.array([[1, 2, 3, 4, 5, 6], [1, 2, 3, 4, 5, 6]])
    tok = np.array([[0, 1, 9, 3, 4, 5], [0, 1, 2, 3, 4, 9]])
    r = O.accept(tok, argmax, np.stack([pid, pid]), np.stack([boff, boff]), np.array([0, 0]), gamma, K, bp)
    assert r["n_accept"].tolist() == [2, 5]
    assert r["n_match"].tolist() == [3, 4]          # Eq. (10): matches over the whole main draft
    assert r["path"].tolist() == [0, 1]
    assert r["bonus"].tolist() == [2, 5]
    assert r["phrase_A"].shape == (2, 1)
