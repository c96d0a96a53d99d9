"""GPU check of ouro_lmhead_argmax_static (the entry point for callers that cannot allocate): same results as
ouro_lmhead_argmax, bit for bit, on calls in a row that share the library's built-in scratch buffer."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import binding as ob, workloads as W
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _both(R, Hd, V, seed, tiled, dtype="bf16"):
    cfg = W.scaled(W.CONFIGS[2], B=1, Hq=Hd // 64, Hkv=Hd // 64, D=64, V=V, dtype=dtype)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    hidden, w = W.make_hidden(cfg, seed, rows=R), W.make_lmhead_weight(cfg, seed)
    h_d = torch.from_numpy(hidden).to(DEV).to(dt)
    w_d = torch.from_numpy(w).to(DEV).to(dt)
    if tiled:
        w_d = ob.ouro_lmhead_pack_w(w_d)
    ref_arg = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    ref_max = torch.full((R,), float("nan"), dtype=torch.float32, device=DEV)
    ob.ouro_lmhead_argmax(h_d, w_d, argmax_out=ref_arg, max_out=ref_max)
    got_arg = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    got_max = torch.full((R,), float("nan"), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ob.ouro_lmhead_argmax_static(h_d, w_d, got_arg, got_max)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before            # the call took nothing from the caching allocator either
    assert torch.equal(got_arg, ref_arg) and torch.equal(got_max, ref_max)
    ref = O.lmhead_argmax(hidden, w)
    arg = got_arg.cpu().numpy()
    bad = [float(ref["margin"][r]) for r in range(R) if arg[r] != ref["argmax"][r]]
    assert all(m < 1e-3 for m in bad), bad


def test_static_scratch_matches_the_workspace_entry_point_on_calls_in_a_row():
    """A large call (the batched workload's shape: 512 rows, the large-tile kernel, 125 slabs), then smaller ones that
    reuse the same buffer with its previous contents still in place (streaming kernels, a ragged vocabulary, fp32)."""
    _both(512, 4096, 32000, 1, True)
    _both(64, 512, 3000, 2, False)
    _both(128, 320, 1025, 3, True)
    _both(16, 256, 1000, 4, False, dtype="f32")
    _both(512, 4096, 32000, 5, False)
