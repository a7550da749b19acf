"""Random shapes through both forms of the selection (fixed seeds: a regression net over shapes nobody thought of).
Every case runs check_compact of test_gpu_compact_selection: the bytes against their definition, the statistics, the
vote bounds against the dense votes and the oracle's, the index set against the oracle's (1e-6 band rule) and against
the five-call form's."""
import math

import numpy as np
import pytest

import workloads as W
from test_gpu_compact_selection import check_compact, make_layer, gpu   # noqa: F401  (gpu is a fixture)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def supported(H_kv, G, P):
    hb = min(H_kv, 8)
    return H_kv * G <= 128 and (P == 1 or (P * hb) % 8 == 0)


def draw_case(rng, matrix_core):
    while True:
        dtype = W.BF16 if (matrix_core or rng.random() < 0.75) else W.F32
        H_kv = int(rng.choice([1, 2, 4, 8, 16]))
        G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        P = int(rng.choice([1, 2, 4, 16, 16, 16]))
        if not supported(H_kv, G, P):
            continue
        if matrix_core and not ((3 <= G <= 4 and H_kv >= 8) or (5 <= G <= 8 and H_kv == 4)):
            continue
        D = int(rng.choice([64, 128]))
        B = int(rng.choice([1, 1, 2, 3]))
        top = 20000 if matrix_core else 6000
        lens = [int(rng.choice([0, 1, 31, 32, 33, 500, 1000, 2047, 2048, 2049, 3000, 5000, 7777])) if rng.random() < 0.5
                else int(rng.integers(1, top)) for _ in range(B)]
        if max(lens) == 0:
            lens[0] = 100
        k = int(rng.choice([2, 64, 500, 2048])) if matrix_core else int(rng.choice([1, 16, 100, 256, 1000]))
        ni = int(rng.choice([0, 0, 0, 4, 128])); nl = int(rng.choice([0, 0, 0, 16, 512]))
        scale = float(rng.choice([1.0, 1.0, 1.0 / math.sqrt(D), 0.3]))
        beta = float(rng.choice([0.0, 2.5, 6.0]))
        return dict(dtype=dtype, H=H_kv * G, H_kv=H_kv, D=D, P=P, B=B, seq_lens=lens, k=k, beta=beta,
                    planted_per_head=0, seed=int(rng.integers(1, 1 << 30))), ni, nl, scale


@pytest.mark.parametrize("seed,matrix_core,cases", [(11, False, 60), (12, True, 40)])
def test_random_shapes(gpu, seed, matrix_core, cases):
    rng = np.random.default_rng(seed)
    for n in range(cases):
        kw, ni, nl, scale = draw_case(rng, matrix_core)
        print("random shape", seed, n, kw, ni, nl, round(scale, 4), flush=True)
        w = W.make_workload("random", **kw)
        layer, q = make_layer(w, num_initial=ni, num_local=nl)
        check_compact(w, layer, q, score_scale=scale, label="seed%d case%d" % (seed, n))
