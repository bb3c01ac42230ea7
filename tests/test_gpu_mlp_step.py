"""GPU test of gpd_mlp_step, the whole training iteration of a small-batch coded MLP with the
master's work between two coded products fused into one launch: it must leave bit for bit the
coded weights, activations and errors that the per-layer gpd_coded_layer_step calls leave (the
parity of those with the oracle is in test_gpu_layer.py and test_gpu_full_configs.py), and the
trajectory must track the oracle's plain SGD."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from paper_1811_10751_amd.mlp import CodedMLP
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu

CASES = [
    # sizes, batch, m, n, P
    ((96, 128, 64, 10), 1, 4, 2, 24),      # the batch-1 workload's code at a small size; 10 outputs, m = 4: padded
    ((96, 128, 64, 10), 4, 2, 4, 32),
    ((50, 70, 33, 7), 8, 2, 4, 20),        # ragged everywhere, widest batch of the path
    ((50, 70, 33, 7), 2, 3, 5, 64),        # 64 nodes
    ((20, 10), 2, 2, 2, 12),               # a single layer
    ((2000, 1100, 600), 1, 4, 2, 24),      # several tiles per stage, more than one chunk of 64 rows
]


@pytest.mark.parametrize("sizes,batch,m,n,P", CASES)
def test_fused_iteration_equals_the_per_layer_calls(sizes, batch, m, n, P):
    say("mlp step", sizes, batch, m, n, P)
    nl = len(sizes) - 1
    rng = np.random.default_rng(sum(sizes) + batch)
    Ws = [(rng.standard_normal((sizes[l + 1], sizes[l])) / np.sqrt(sizes[l])).astype(np.float32) for l in range(nl)]
    fused = CodedMLP(sizes, batch, m, n, 1, 1, P)
    plain = CodedMLP(sizes, batch, m, n, 1, 1, P)
    plain.fused = False                                   # per-layer gpd_coded_layer_step calls only
    for mlp in (fused, plain):
        mlp.encode_weights([to_dev(w) for w in Ws])
    Ws_o = [w.astype(np.float64) for w in Ws]
    eta, decay = 0.5, 0.01
    # how much the decoders of this code amplify fp32 rounding (long codes on few useful coefficients
    # are ill-conditioned: the bar against the exact trajectory scales with it)
    amp = 1.0
    for l in range(nl):
        olp = O.make_layer_plan(sizes[l + 1], sizes[l], batch, m, n, 1, 1, P, "auto")
        Db = np.linalg.pinv(O.vandermonde(olp.points, olp.Kb))
        amp = max(amp, O.amplification(olp.fwd, None, "lsq_all"), max(np.linalg.norm(Db[int(e)]) for e in olp.eCb.ravel()))
    tol = max(1e-3, 2e-5 * amp)
    for step in range(4):
        X, Y = WL.mlp_batch(3, step, sizes[0], sizes[-1], batch)
        y_f, _ = fused.step(to_dev(X), to_dev(Y), eta, decay)
        y_p, _ = plain.step(to_dev(X), to_dev(Y), eta, decay)
        torch.cuda.synchronize()
        assert fused.fused is True
        assert torch.equal(y_f, y_p)
        for l in range(nl):
            assert torch.equal(fused.acts[l + 1], plain.acts[l + 1]), (step, l)
            assert torch.equal(fused.deltas[l], plain.deltas[l]), (step, l)
            assert torch.equal(fused.Wts[l], plain.Wts[l]), (step, l)
        Ws_o, y_o, _ = O.mlp_uncoded_step(Ws_o, X, Y, np.float32(eta), np.float32(decay))
        err = rel_fro(to_np(y_f), y_o)
        say("  step %d: output vs plain fp64 SGD %.3g (amplification %.3g)" % (step, err, amp))
        assert err < tol
    for W_dec, W_ref in zip(fused.decode_weights(), Ws_o):
        assert rel_fro(to_np(W_dec), W_ref) < tol


def test_what_the_fused_path_does_not_cover_falls_back():
    # batch 24 goes through the matrix-core products: gpd_mlp_step declines, the iteration runs
    # through the per-layer calls and gives the same result as before
    sizes, batch = (96, 128, 64, 10), 24
    mlp = CodedMLP(sizes, batch, 2, 4, 1, 1, 32)
    Ws = WL.mlp_init(sizes, seed=2)
    mlp.encode_weights([to_dev((w * 8).astype(np.float32)) for w in Ws])
    X, Y = WL.mlp_batch(2, 0, sizes[0], sizes[-1], batch)
    yhat, _ = mlp.step(to_dev(X), to_dev(Y), 0.5)
    assert mlp.fused is False and yhat.shape == (10, batch)
    # a network whose layers do not chain is an error of the caller's
    L1 = G.gpd_layer_create(8, 16, 1, 2, 2, 1, 1, 12)
    L2 = G.gpd_layer_create(4, 9, 1, 2, 2, 1, 1, 12)
    Wt1 = G.gpd_layer_encode_weights(L1, torch.zeros((8, 16), device=DEV))
    Wt2 = G.gpd_layer_encode_weights(L2, torch.zeros((4, 9), device=DEV))
    acts = [torch.zeros((8, 1), device=DEV), torch.zeros((4, 1), device=DEV)]
    assert G.gpd_mlp_step([L1, L2], [Wt1, Wt2], torch.zeros((16, 1), device=DEV), torch.zeros((4, 1), device=DEV),
                          0.1, 0.0, acts) is False
