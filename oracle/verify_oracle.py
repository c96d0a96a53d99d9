"""CPU oracle for the Ouroboros verification step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what one verification pass computes
(Ouroboros, Sec. 2 Eq. (2)-(3) and Sec. 3.2 Eq. (7)-(9)): every token of a draft
block -- a main draft d_1..gamma plus K candidate phrase suffixes -- is scored by
the target model in one pass, each row conditioned on exactly the tokens its own
lengthened draft would put before it; the per-row greedy prediction is compared
with the draft, and the longest accepted prefix is chosen.

It shares no code with the HIP library and must never be imported by the product
path: only tests, the smoke check and the bench's cpu_baseline leg call it.

Pins (tests/test_oracle_*.py): visibility against a hand-written mask derived
from Eq. (8) (tests/golden), against one-by-one causal verification of each
lengthened draft (Sec. 3.2: the masked pass replaces verifying them one by one),
probe/closed-form cases; attention against a library SDPA on textbook cases and
the log-sum-exp split identity; LM head against planted winners and ties;
acceptance against hand-worked traces (tests/golden), exhaustive path
enumeration, and the lossless replay property of Eq. (4); the phrase-pool
by-products against a hand-worked example, a regular-expression scan of the match
string and the definition of Eq. (10); the commit of accepted
tokens against a hand-worked example (tests/golden), a concatenation written
with library routines, and the property that a committed cache gives the next
step the context of the accepted draft; the chained step (verify_step) against
planted greedy tokens computed through a library attention routine and against
the all-correct-draft invariant.  No function here is "parity unpinned".

Conventions (readings of points the paper leaves open):
  * Block token t carries (pid[t], boff[t]).  pid 0 = main draft, main token i
    has boff = i.  Phrase j >= 1 occupies a contiguous ascending index range;
    all of its tokens carry boff = b_j, the 0-based main index the phrase hangs
    off.  The paper's layout is b_j = gamma-1 for all j (phrases start with
    d_gamma).  b_j = -1 means the phrase hangs off the last cached token.
  * Eq. (8) writes the phrase index range loosely (j from 2, i to beta+1); the
    reading here is j = 1..K, and a phrase contributes beta-1 block tokens
    p^j_2..p^j_beta, the shared first token p^j_1 = d_gamma not being repeated.
  * Rows are next-token predictions: the row of block token t is the target's
    distribution given the prefix, t's ancestors and t itself.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

ROOT = -1  # parent of a token that hangs directly off the cached prefix


# --------------------------------------------------------------------------- #
# Tree structure of the block (Eq. (7): K lengthened drafts sharing d_1..gamma)
# --------------------------------------------------------------------------- #
def parents(pid: np.ndarray, boff: np.ndarray) -> np.ndarray:
    """parent[t] = block index of the token that precedes t in its own lengthened draft.

    Main token i follows main token i-1 (main 0 follows the prefix).  The first
    token of phrase j follows main token b_j; every later phrase token follows
    the previous token of the same phrase.
    """
    pid = np.asarray(pid).astype(np.int64)
    boff = np.asarray(boff).astype(np.int64)
    T = pid.shape[0]
    par = np.empty(T, dtype=np.int64)
    for t in range(T):
        if pid[t] == 0:
            par[t] = t - 1 if t > 0 else ROOT
        elif t > 0 and pid[t - 1] == pid[t]:
            par[t] = t - 1
        else:
            par[t] = boff[t] if boff[t] >= 0 else ROOT
    return par


def block_visibility(pid: np.ndarray, boff: np.ndarray) -> np.ndarray:
    """Dense [T, T] boolean: vis[q, k] iff block token k is in the conditioning set of row q.

    Eq. (2) / Eq. (8): the row for token q is conditioned on the prefix, on the
    tokens that precede q in q's own lengthened draft, and on q itself (q is the
    newest input token when its next-token distribution is computed).  That set
    is q plus its chain of ancestors; nothing else in the block is visible.
    """
    par = parents(pid, boff)
    T = par.shape[0]
    vis = np.zeros((T, T), dtype=bool)
    for q in range(T):
        t = q
        while t != ROOT:
            vis[q, t] = True
            t = par[t]
    return vis


def dense_mask(pid: np.ndarray, boff: np.ndarray, L: int) -> np.ndarray:
    """[T, L+T] mask over [cached prefix | block]: every cached key is visible to every row."""
    T = np.asarray(pid).shape[0]
    m = np.ones((T, L + T), dtype=bool)
    m[:, L:] = block_visibility(pid, boff)
    return m


# --------------------------------------------------------------------------- #
# Draft-block attention (the attention inside the single verifying forward, Sec. 3.2)
# --------------------------------------------------------------------------- #
def masked_softmax_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                             mask: np.ndarray, scale: float):
    """softmax(scale * q k^T restricted to mask) v for one head, fp64.

    q [T, D], k/v [N, D], mask [T, N] bool.  Returns (out [T, D], lse [T]) where
    lse is the natural-log of the softmax denominator (before max subtraction).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    s = (q @ k.T) * float(scale)
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    den = e.sum(axis=1, keepdims=True)
    out = (e / den) @ v
    lse = (m + np.log(den))[:, 0]
    return out, lse


def verify_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                     cu_seqlens: np.ndarray, k_blk: np.ndarray, v_blk: np.ndarray,
                     pid: np.ndarray, boff: np.ndarray,
                     scale: Optional[float] = None,
                     heads: Optional[list] = None,
                     seq_len: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Attention of every block row over [its sequence's cache | visible block tokens].

    q [B,T,Hq,D]; k_cache/v_cache [sum L_b, Hkv, D] with sequence b at rows
    cu_seqlens[b]:cu_seqlens[b+1]; k_blk/v_blk [B,T,Hkv,D]; pid/boff [B,T].
    With ``seq_len`` [B] only the first seq_len[b] rows of sequence b's region are
    cached tokens (the rest of the region is room for tokens accepted later).
    Query head h reads key/value head h // (Hq // Hkv) (consecutive query heads
    share a KV head).  scale defaults to 1/sqrt(D).  ``heads`` optionally limits
    the computation to a list of (b, h) pairs (others are left NaN) so that large
    workloads can be checked on a sample.
    Returns out [B,T,Hq,D] fp64 and lse [B,Hq,T] fp64.
    """
    B, T, Hq, D = q.shape
    Hkv = k_blk.shape[2]
    group = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.full((B, T, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((B, Hq, T), np.nan, dtype=np.float64)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    masks = {}
    for (b, h) in todo:
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        if seq_len is not None:
            hi = lo + int(seq_len[b])
        if b not in masks:
            masks[b] = dense_mask(pid[b], boff[b], hi - lo)
        g = h // group
        keys = np.concatenate([k_cache[lo:hi, g, :], k_blk[b, :, g, :]], axis=0)
        vals = np.concatenate([v_cache[lo:hi, g, :], v_blk[b, :, g, :]], axis=0)
        o, l = masked_softmax_attention(q[b, :, h, :], keys, vals, masks[b], scale)
        out[b, :, h, :] = o
        lse[b, h, :] = l
    return {"out": out, "lse": lse}


# --------------------------------------------------------------------------- #
# LM head + greedy pick (Eq. (2) with the greedy setting of Sec. 4)
# --------------------------------------------------------------------------- #
def lmhead_argmax(hidden: np.ndarray, w: np.ndarray) -> Dict[str, np.ndarray]:
    """logits[r, v] = sum_k hidden[r, k] * w[v, k] in fp64; greedy token per row.

    hidden [R, Hd]; w [V, Hd].  Ties go to the smallest token id.  Also returns
    the best and second-best logit and their difference (margin) per row.
    """
    logits = np.asarray(hidden, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    R, V = logits.shape
    arg = np.argmax(logits, axis=1).astype(np.int32)      # first occurrence of the maximum
    top1 = logits[np.arange(R), arg]
    if V > 1:
        rest = logits.copy()
        rest[np.arange(R), arg] = -np.inf
        top2 = rest.max(axis=1)
    else:
        top2 = np.full(R, -np.inf)
    return {"argmax": arg, "top1": top1, "top2": top2, "margin": top1 - top2}


# --------------------------------------------------------------------------- #
# Acceptance (Eq. (3), Eq. (9), and the selection rule that follows Eq. (9))
# --------------------------------------------------------------------------- #
def expected_tokens(argmax: np.ndarray, pid: np.ndarray, boff: np.ndarray,
                    root_pred: Optional[int]) -> np.ndarray:
    """v for each block position: the target's greedy token at that position, i.e. the
    prediction made by the row of the position's parent (root_pred for a child of the prefix).
    With root_pred None a child of the prefix has no check; -1 is returned there."""
    par = parents(pid, boff)
    T = par.shape[0]
    exp = np.empty(T, dtype=np.int64)
    for t in range(T):
        if par[t] == ROOT:
            exp[t] = -1 if root_pred is None else int(root_pred)
        else:
            exp[t] = int(argmax[par[t]])
    return exp


def accept_one(tok: np.ndarray, argmax: np.ndarray, pid: np.ndarray, boff: np.ndarray,
               root_pred: Optional[int], gamma: int, K: int, beta_p: int) -> Dict[str, object]:
    """Longest accepted prefix for one sequence.

    A (Eq. (3)): walk the main draft from its first token, stop at the first token that
    differs from the target's prediction for that position.  A-hat'_j (Eq. (9)): the same
    walk along phrase j's beta_p block tokens.  A phrase is usable only if the draft up
    to and including its branch token is accepted (the paper states the b_j = gamma-1
    case: the draft must be fully accepted); among the main draft alone and the usable
    phrases the longest total wins, the lowest path id on ties.  The token after the
    accepted run (bonus) is the prediction of the last accepted row.

    root_pred None: main token 0 is the already-accepted last token of the sequence
    (no check; it counts as accepted).  Nothing else is accepted without a check: Eq. (4)
    needs every accepted token to equal a prediction of the target.  A phrase that hangs
    off the prefix (b_j = -1) then has no prediction its first token could be compared
    with; that token counts as a mismatch, so the phrase's run is empty and it never wins.
    """
    tok = np.asarray(tok).astype(np.int64)
    argmax = np.asarray(argmax).astype(np.int64)
    T = gamma + K * beta_p
    assert tok.shape[0] == T
    v = expected_tokens(argmax, pid, boff, root_pred)
    par = parents(pid, boff)

    def matches(t: int) -> bool:
        if par[t] == ROOT and root_pred is None:
            return t == 0                    # no prediction to check against: only main token 0 is pre-accepted
        return bool(tok[t] == v[t])

    A = 0
    while A < gamma and matches(A):
        A += 1
    phrase_A = np.zeros(K, dtype=np.int32)
    best_len, best_path = A, 0
    for j in range(1, K + 1):
        lo = gamma + (j - 1) * beta_p
        bj = int(boff[lo])
        n = 0
        while n < beta_p and matches(lo + n):
            n += 1
        phrase_A[j - 1] = n
        if A >= bj + 1:
            total = bj + 1 + n
            if total > best_len:
                best_len, best_path = total, j
    idx = np.full(gamma + beta_p, -1, dtype=np.int32)
    if best_path == 0:
        accepted = list(range(A))
    else:
        lo = gamma + (best_path - 1) * beta_p
        bj = int(boff[lo])
        accepted = list(range(bj + 1)) + [lo + i for i in range(int(phrase_A[best_path - 1]))]
    idx[: len(accepted)] = accepted
    if accepted:
        bonus = int(argmax[accepted[-1]])
    else:
        bonus = -1 if root_pred is None else int(root_pred)
    n_match = int(sum(matches(i) for i in range(gamma)))   # #Match of Eq. (10), over the main draft
    return {"n_accept": len(accepted), "path": best_path, "bonus": bonus, "accept_idx": idx,
            "main_A": A, "phrase_A": phrase_A, "n_match": n_match}


def accept(tok: np.ndarray, argmax: np.ndarray, pid: np.ndarray, boff: np.ndarray,
           root_pred: Optional[np.ndarray], gamma: int, K: int, beta_p: int) -> Dict[str, np.ndarray]:
    """Per-sequence acceptance over a batch: tok/argmax/pid/boff [B,T], root_pred [B] or None."""
    B = tok.shape[0]
    res = [accept_one(tok[b], argmax[b], pid[b], boff[b],
                      None if root_pred is None else int(root_pred[b]), gamma, K, beta_p)
           for b in range(B)]
    return {
        "n_accept": np.array([r["n_accept"] for r in res], dtype=np.int32),
        "path": np.array([r["path"] for r in res], dtype=np.int32),
        "bonus": np.array([r["bonus"] for r in res], dtype=np.int32),
        "accept_idx": np.stack([r["accept_idx"] for r in res]).astype(np.int32),
        "main_A": np.array([r["main_A"] for r in res], dtype=np.int32),
        "phrase_A": np.stack([r["phrase_A"] for r in res]).astype(np.int32).reshape(B, K),
        "n_match": np.array([r["n_match"] for r in res], dtype=np.int32),
    }


# --------------------------------------------------------------------------- #
# What verification leaves for the phrase pool (Sec. 3.3: Eq. (10) and the two
# paragraphs after it)
# --------------------------------------------------------------------------- #
def pool_byproducts_one(tok: np.ndarray, argmax: np.ndarray, pid: np.ndarray, boff: np.ndarray,
                        root_pred: Optional[int], gamma: int, K: int, beta_p: int) -> Dict[str, object]:
    """By-products of one sequence's verification.

    match[t] = [tok[t] == v[t]] for every block position, v[t] being the target's greedy token at that
    position (the prediction of the row of t's parent); its sum over the main draft is #Match of Eq. (10).
    With no root_pred, main token 0 counts as a match and the first token of a phrase that hangs off the
    prefix as a mismatch, as in accept_one.

    Segments: the maximal runs of consecutive matching positions inside the discarded part of the main
    draft, d_{A+1..gamma} (0-based positions >= A; position A itself is the first mismatch), as
    (start, length) pairs in ascending order: the sub-segments of the discarded draft that agree with
    the verification result.  Which of them are worth keeping (a minimum length) is the caller's policy.

    Repaired phrases: for every phrase o, (p^o_1, v^o_2..beta): its first token, which is the main-draft
    token at its branch point (-1 for a phrase that hangs off the prefix: that token is not in the block),
    followed by the target's greedy tokens at the phrase's beta_p block positions.  The caller replaces
    the phrases it did not use (o != path) with these.
    """
    tok = np.asarray(tok).astype(np.int64)
    T = gamma + K * beta_p
    v = expected_tokens(np.asarray(argmax).astype(np.int64), pid, boff, root_pred)
    par = parents(pid, boff)
    match = np.zeros(T, dtype=np.uint8)
    for t in range(T):
        if par[t] == ROOT and root_pred is None:
            match[t] = 1 if t == 0 else 0
        else:
            match[t] = 1 if tok[t] == v[t] else 0
    A = 0
    while A < gamma and match[A]:
        A += 1
    starts, lens = [], []
    i = A
    while i < gamma:
        if match[i]:
            j = i
            while j < gamma and match[j]:
                j += 1
            starts.append(i)
            lens.append(j - i)
            i = j
        else:
            i += 1
    nmax = max(1, (gamma + 1) // 2)
    seg_start = np.full(nmax, -1, dtype=np.int32)
    seg_len = np.zeros(nmax, dtype=np.int32)
    seg_start[: len(starts)] = starts
    seg_len[: len(lens)] = lens
    repaired = np.full((K, beta_p + 1), -1, dtype=np.int32)
    for o in range(1, K + 1):
        lo = gamma + (o - 1) * beta_p
        bo = int(boff[lo])
        repaired[o - 1, 0] = tok[bo] if bo >= 0 else -1
        for i in range(beta_p):
            repaired[o - 1, 1 + i] = v[lo + i]
    return {"match": match, "n_seg": len(starts), "seg_start": seg_start, "seg_len": seg_len, "repaired": repaired}


def pool_byproducts(tok: np.ndarray, argmax: np.ndarray, pid: np.ndarray, boff: np.ndarray,
                    root_pred: Optional[np.ndarray], gamma: int, K: int, beta_p: int) -> Dict[str, np.ndarray]:
    """Batch form of pool_byproducts_one: match [B,T] uint8, n_seg [B], seg_start/seg_len
    [B, ceil(gamma/2)] (-1 / 0 padded), repaired [B,K,beta_p+1]."""
    B = tok.shape[0]
    res = [pool_byproducts_one(tok[b], argmax[b], pid[b], boff[b],
                               None if root_pred is None else int(root_pred[b]), gamma, K, beta_p)
           for b in range(B)]
    return {
        "match": np.stack([r["match"] for r in res]),
        "n_seg": np.array([r["n_seg"] for r in res], dtype=np.int32),
        "seg_start": np.stack([r["seg_start"] for r in res]),
        "seg_len": np.stack([r["seg_len"] for r in res]),
        "repaired": np.stack([r["repaired"] for r in res]).reshape(B, K, beta_p + 1),
    }


# --------------------------------------------------------------------------- #
# Keeping the accepted tokens (the sentence after Eq. (3): d_1..A are accepted and
# the rest of the draft is discarded; after Eq. (9): d_1..gamma, p^j_2..Ahat^j)
# --------------------------------------------------------------------------- #
def kv_commit(k_cache: np.ndarray, v_cache: np.ndarray, cu_seqlens: np.ndarray, seq_len: np.ndarray,
              k_blk: np.ndarray, v_blk: np.ndarray, accept_idx: np.ndarray,
              n_accept: np.ndarray) -> Dict[str, np.ndarray]:
    """Append the keys/values of the accepted block tokens to each sequence's cache.

    Sequence b owns rows cu_seqlens[b]:cu_seqlens[b+1] of k_cache/v_cache
    [rows, Hkv, D]; the first seq_len[b] of them are its cached tokens.  The
    accepted block tokens accept_idx[b, 0:n_accept[b]] (block indices, in the order
    of the accepted draft) become cached tokens seq_len[b], seq_len[b]+1, ...; all
    other block tokens are dropped.  A sequence whose region cannot take its
    accepted tokens is left untouched and flagged.
    Returns new k_cache, v_cache, seq_len and overflow [B] (0/1); inputs are not modified.
    """
    k_new, v_new = k_cache.copy(), v_cache.copy()
    len_new = np.array(seq_len, dtype=np.int64).copy()
    B = k_blk.shape[0]
    overflow = np.zeros(B, dtype=np.int32)
    for b in range(B):
        start = int(cu_seqlens[b])
        room = int(cu_seqlens[b + 1]) - start
        have = int(seq_len[b])
        na = int(n_accept[b])
        if have + na > room:
            overflow[b] = 1
            continue
        for i in range(na):
            t = int(accept_idx[b, i])
            k_new[start + have + i] = k_blk[b, t]
            v_new[start + have + i] = v_blk[b, t]
        len_new[b] = have + na
    return {"k_cache": k_new, "v_cache": v_new, "seq_len": len_new, "overflow": overflow}


# --------------------------------------------------------------------------- #
# The whole verification step, chained
# --------------------------------------------------------------------------- #
def verify_step(inp: Dict[str, np.ndarray], w: np.ndarray, tok,
                root_pred: Optional[np.ndarray], gamma: int, K: int, beta_p: int,
                hidden_round=None) -> Dict[str, np.ndarray]:
    """attention -> LM head -> argmax -> acceptance on one batch of inputs (Sec. 3.2: one forward of the
    target over the whole block, then Eq. (3) / Eq. (9)).

    The hidden state of block row (b, t) is its attention output with the heads side by side,
    hidden[b*T + t, h*D + d] = out[b, t, h, d].  ``hidden_round`` optionally maps that fp64 array to the values
    the LM head is fed (e.g. rounding to bf16, which is what a bf16 attention output stores).
    ``tok`` is the draft, int [B, T], or a function that builds it from the chain's own greedy tokens
    [B, T] (workloads whose drafts are partly "the token the target will predict" need those first).
    """
    att = verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                           inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])
    B, T, Hq, D = att["out"].shape
    hidden = att["out"].reshape(B * T, Hq * D)
    if hidden_round is not None:
        hidden = hidden_round(hidden)
    lm = lmhead_argmax(hidden, w)
    amax = lm["argmax"].reshape(B, T)
    if callable(tok):
        tok = tok(amax)
    acc = accept(tok, amax, inp["pid"], inp["boff"], root_pred, gamma, K, beta_p)
    return {"attn": att, "hidden": hidden, "lm": lm, "tok": tok, "accept": acc}
