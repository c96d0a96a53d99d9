"""Mutation check of the oracle's pins (CPU only; run by hand: ``python tests/oracle_mutation_check.py``).

Each entry plants one plausible one-line mistake in a COPY of the oracle (a wrong parent, a dropped scale, a
transposed operand, an off-by-one, a wrong tie rule, ...) and runs the ``-m "not gpu"`` tests against that copy:
a mistake that no pin notices would print SURVIVED.  Nothing here touches the GPU or the working tree.
"""
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = [
    ("oracle/verify_oracle.py", "par[t] = boff[t] if boff[t] >= 0 else ROOT", "par[t] = boff[t]-1 if boff[t] >= 1 else ROOT"),
    ("oracle/verify_oracle.py", "s = (q @ k.T) * float(scale)", "s = (q @ k.T)"),
    ("oracle/verify_oracle.py", "scale = 1.0 / np.sqrt(D)", "scale = 1.0 / D"),
    ("oracle/verify_oracle.py", "g = h // group", "g = h % Hkv"),
    ("oracle/verify_oracle.py", "@ np.asarray(w, dtype=np.float64).T", "@ np.asarray(w, dtype=np.float64).T * -1"),
    ("oracle/verify_oracle.py", "if A >= bj + 1:", "if A >= bj:"),
    ("oracle/verify_oracle.py", "total = bj + 1 + n", "total = bj + n"),
    ("oracle/verify_oracle.py", "if total > best_len:", "if total >= best_len:"),
    ("oracle/verify_oracle.py", "bonus = int(argmax[accepted[-1]])", "bonus = int(argmax[accepted[0]])"),
    ("oracle/verify_oracle.py", "lse = (m + np.log(den))[:, 0]", "lse = (np.log(den))[:, 0]"),
    ("oracle/verify_oracle.py", "out = (e / den) @ v", "out = e @ v"),
    ("oracle/verify_oracle.py", "elif t > 0 and pid[t - 1] == pid[t]:", "elif t > 0 and pid[t - 1] != 0:"),
    ("oracle/verify_oracle.py", "hi = lo + int(seq_len[b])", "hi = lo + int(seq_len[b]) + 1"),
    ("oracle/verify_oracle.py", "return t == 0                    # no prediction", "return True                      # no prediction"),
    ("oracle/verify_oracle.py", "match[t] = 1 if t == 0 else 0", "match[t] = 1"),
    # the chained step
    ("oracle/verify_oracle.py", "hidden = att[\"out\"].reshape(B * T, Hq * D)", "hidden = att[\"out\"].transpose(0, 1, 3, 2).reshape(B * T, Hq * D)"),
    ("oracle/verify_oracle.py", "amax = lm[\"argmax\"].reshape(B, T)", "amax = lm[\"argmax\"].reshape(T, B).T"),
    # commit of accepted tokens
    ("oracle/verify_oracle.py", "k_new[start + have + i] = k_blk[b, t]", "k_new[start + have + i] = k_blk[b, i]"),
    ("oracle/verify_oracle.py", "v_new[start + have + i] = v_blk[b, t]", "v_new[start + have + i] = k_blk[b, t]"),
    ("oracle/verify_oracle.py", "if have + na > room:", "if have + na >= room:"),
    ("oracle/verify_oracle.py", "len_new[b] = have + na", "len_new[b] = have + na + 1"),
    # phrase-pool by-products
    ("oracle/verify_oracle.py", "    i = A\n    while i < gamma:", "    i = 0\n    while i < gamma:"),
    ("oracle/verify_oracle.py", "repaired[o - 1, 0] = tok[bo] if bo >= 0 else -1", "repaired[o - 1, 0] = tok[lo]"),
    ("oracle/verify_oracle.py", "repaired[o - 1, 1 + i] = v[lo + i]", "repaired[o - 1, 1 + i] = tok[lo + i]"),
    # layer oracle
    ("oracle/layer_oracle.py", "n += 1\n            u = par[u]", "u = par[u]"),
    ("oracle/layer_oracle.py", "inv = base ** (-2.0 * np.arange(half) / D)", "inv = base ** (-1.0 * np.arange(half) / D)"),
    ("oracle/layer_oracle.py", "a * c - b * s, b * c + a * s", "a * c + b * s, b * c - a * s"),
    ("oracle/layer_oracle.py", "return x / np.sqrt(ms + eps)", "return x / (np.sqrt(ms) + eps)"),
    ("oracle/layer_oracle.py", "out[r] = (ws * xs[r][None, :]).sum(axis=1)", "out[r] = (ws * xs[r][None, :]).sum(axis=1)[::-1]"),
    ("oracle/layer_oracle.py", "return g / (1.0 + np.exp(-g)) * u", "return u / (1.0 + np.exp(-u)) * g"),
]


def main() -> int:
    survived = 0
    with tempfile.TemporaryDirectory() as tmp:
        for sub in ("oracle", "tests", "paper_2402_13720_amd", "include"):
            shutil.copytree(os.path.join(ROOT, sub), os.path.join(tmp, sub),
                            ignore=shutil.ignore_patterns("__pycache__", "_build"))
        for path, good, bad in MUTATIONS:
            f = os.path.join(tmp, path)
            src = open(f).read()
            if good not in src:
                print("STALE    | %s: %r not found" % (path, good))
                survived += 1
                continue
            open(f, "w").write(src.replace(good, bad, 1))
            r = subprocess.run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                               cwd=tmp, capture_output=True, text=True)
            open(f, "w").write(src)
            killed = r.returncode != 0
            survived += not killed
            print("%-8s | %s: %s" % ("KILLED" if killed else "SURVIVED", path, good.replace("\n", " ")[:70]), flush=True)
    print("%d of %d mutations survived" % (survived, len(MUTATIONS)))
    return 1 if survived else 0


if __name__ == "__main__":
    sys.exit(main())
