"""rtl_sparse_linear_static (the entry point that allocates nothing) against rtl_sparse_linear.

Both run the same kernels in the same order, so the outputs must be identical; the fixed scratch
is shared by all calls on the GPU and keeps the previous call's contents, hence two calls in a row,
the second on a smaller problem, each checked against the workspace-taking entry point and, on
sampled rows, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26632_amd import binding as rtl
from paper_2605_26632_amd import synth
from util import Y_TOL, floored_elem_err, rel_max_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_pair(X, W, comp, bias=None):
    M, N = X.shape[0], W.shape[0]
    Y_ref = rtl.sparse_linear(X, W, bias=bias, comp=comp)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rtl.sparse_linear_static(X, W, Y, bias=bias, comp=comp)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before        # the binding allocated nothing either
    assert torch.equal(Y, Y_ref)
    return Y


def test_static_scratch_entry_point_two_calls_second_smaller():
    # first call: the headline shape (56.6 MB of scratch in use)
    X, W = synth.workload("mlp_down", seed=0, device=DEV)
    assert rtl.sparse_linear_workspace(*[X.shape[0], W.shape[0], X.shape[1]]) <= rtl.STATIC_SCRATCH_BYTES
    Y = run_pair(X, W, rtl.COMP_GROUP)
    rows = np.array([0, 1500, 4095])
    sel = torch.from_numpy(rows).to(DEV)
    ref = oracle.sparse_linear_oracle(synth.bits(X[sel]), synth.bits(W), scope=oracle.GROUP)["Y"]
    y = Y[sel].float().cpu().numpy()
    assert rel_max_err(y, ref) <= Y_TOL and floored_elem_err(y, ref) <= Y_TOL
    # second call: smaller and ragged, other scopes, with a bias; stale scratch contents must not matter
    Xs = synth.activations("laplace_outlier", 333, 640, seed=9, device=DEV)
    Ws = synth.weights(200, 640, seed=10, device=DEV, std=1.0)
    b = synth.bias(200, seed=11, device=DEV, std=2.0)
    for comp in (rtl.COMP_ROW, rtl.COMP_TENSOR, rtl.COMP_GROUP, rtl.COMP_NONE):
        Ys = run_pair(Xs, Ws, comp, bias=b)
        ref = oracle.sparse_linear_oracle(synth.bits(Xs), synth.bits(Ws), bias=synth.bits(b), scope=comp)["Y"]
        y = Ys.float().cpu().numpy()
        assert rel_max_err(y, ref) <= Y_TOL and floored_elem_err(y, ref) <= Y_TOL


def test_static_scratch_entry_point_refuses_oversized_problems():
    L = rtl.lib()
    M, N, K = 16896, 3072, 12288                         # needs 233 MB of scratch
    assert rtl.sparse_linear_workspace(M, N, K) > rtl.STATIC_SCRATCH_BYTES
    X = torch.zeros((8, 64), dtype=torch.bfloat16, device=DEV)      # never touched: refused before any launch
    st = L.rtl_sparse_linear_static(X.data_ptr(), X.data_ptr(), None, X.data_ptr(), M, N, K, K, K, N, 1, 1e-8, None)
    assert st == 4
    # ordinary argument errors are reported as by rtl_sparse_linear
    assert L.rtl_sparse_linear_static(None, X.data_ptr(), None, X.data_ptr(), 8, 8, 64, 64, 64, 8, 1, 1e-8, None) == 1
    assert L.rtl_sparse_linear_static(X.data_ptr(), X.data_ptr(), None, X.data_ptr(), 8, 8, 32, 32, 32, 8, 1, 1e-8, None) == 2
