"""GPU parity of the chained verification step: attention -> LM head + arg-max -> acceptance at the full size of
every workload, each stage checked against the oracle on identical inputs, and the whole chain against the oracle's
own chain with every differing row accounted for (see chain_util)."""
import pytest

from paper_2402_13720_amd import workloads as W
from chain_util import format_report, run_chain

pytestmark = pytest.mark.gpu


def _chain(cfg, seed, **kw):
    rep = run_chain(cfg, seed, **kw)
    print(format_report(rep), flush=True)
    return rep


def test_config1_chain():
    for trial in range(3):
        _chain(W.CONFIGS[1], W.seed_for(1, trial))


@pytest.mark.parametrize("cfg_id", [2, 3, 4, 5])
def test_full_size_chain(cfg_id):
    _chain(W.CONFIGS[cfg_id], W.seed_for(cfg_id))


def test_config2_chain_paper_layout_row_major_operands():
    """Every phrase hanging off the last main token (the paper's own layout), caches token-major, W row-major."""
    _chain(W.CONFIGS[2], W.seed_for(2, 1), branch="last", tiled=False, head_major=False)


def test_small_batched_varlen_chain():
    cfg = W.scaled(W.CONFIGS[5], B=4, Hq=4, Hkv=4, L=(100, 900), V=3000)
    _chain(cfg, 99, branch="any")
