"""Seeded sweep over random valid shapes: the stage-wise parity tests of the matmul path and of the
layer step (fp32, bf16 and split workers) called with shapes nobody picked by hand: block grids
from 1 x 1 to 4 x 4, ragged sizes, per-node batches on and off the streaming path, codes from
P = K (no redundancy) to P = K + 8."""
import numpy as np
import pytest

from oracle import gpd_oracle as O
import test_gpu_bf16 as TB
import test_gpu_layer as TL
import test_gpu_matmul as TM
import test_gpu_split as TS
from gpu_util import say

pytestmark = pytest.mark.gpu


def cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    it = 0
    while len(out) < count:
        kind = it % 6
        it += 1
        if kind in (0, 3, 4):
            m, n, d = (int(rng.integers(1, 4)) for _ in range(3))
            K = m * n * d + n - 1
            if K > 14:
                continue
            P = K + int(rng.integers(0, 7))
            hi = 520 if (kind != 0 and rng.random() < 0.5) else 200
            N1, N0, Nc = (q * int(rng.integers(1, hi // q + 1)) for q in (m, n, d))
            out.append((kind, (N1, N0, Nc, m, n, d, P)))
        else:
            m, n = int(rng.integers(1, 5)), int(rng.integers(1, 5))
            d1, d2 = int(rng.integers(1, 3)), int(rng.integers(1, 3))
            pool = [1, 2, 4, 8, 16, 24, 48] if kind == 1 else [1, 2, 4, 8, 6, 12, 24, 64, 128, 192]
            batch = int(rng.choice(pool))
            if batch % d1 or batch % d2:
                d1 = d2 = 1
            N_out, N_in = int(rng.integers(3, 400)), int(rng.integers(3, 400))
            lp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, 64, "auto")
            K = max(lp.Kf, lp.Kb)
            if K > 14:
                continue
            out.append((kind, (N_out, N_in, batch, m, n, d1, d2, K + int(rng.integers(0, 9)))))
    return out


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes(seed):
    for kind, a in cases(seed, 36):
        say("sweep", seed, kind, a)
        if kind == 0:
            TM.test_encode_products_decode_stagewise(*a, "u=v^n")
        elif kind == 3:
            TB.test_bf16_matmul_stagewise(*a)
        elif kind == 4:
            TS.test_split_products_are_fp32_accurate(*a)
        elif kind == 1:
            TL.test_layer_forward_backward_update(*a, "auto")
        elif kind == 2:
            TB.test_bf16_layer_stagewise(*a)
        else:
            TS.test_split_layer_step(*a)
