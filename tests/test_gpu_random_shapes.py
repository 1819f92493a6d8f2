"""Seeded sweep of small random stage shapes (both dtypes, both orders, every stage kind and flag) against the
float64 oracle: shapes the fixed cases do not name -- odd head counts, ragged ffn widths, sequence lengths that
miss the MFMA kernels' tile sizes, K anywhere in 1..M."""
import random

import numpy as np
import pytest

from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I
from tests.stage_util import compare, make_inputs, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _cases(seed, n, big):
    rng = random.Random(seed)
    out = []
    while len(out) < n:
        dtype = rng.choice(["f32", "bf16"])
        d = rng.choice([64, 64, 32, 16] if big else [8, 16, 32, 64])
        A = rng.choice([2, 3, 4, 6] if big else [1, 2, 3, 4])
        H = d * A
        F = rng.choice([H, 2 * H, 4 * H, H + 8, 3 * H - 8, 2 * H + 4])
        if dtype == "bf16" and (H % 8 or F % 8):
            continue                       # refused by the library: bf16 rows are read 16 bytes at a time
        s = rng.choice([64, 128, 192, 256, 40] if big else [8, 16, 24, 40, 64, 128])
        b, L = rng.choice([1, 2, 3]), rng.choice([1, 2, 3])
        M = rng.randint(1, 5)
        K = rng.randint(1, M)
        emb = rng.random() < 0.25
        head = (not emb) and rng.random() < 0.3
        cfg = I.StageConfig(L, H, A, F, s, b, M, K, dtype, has_embedding=emb, has_mlm_head=head,
                            vocab=rng.choice([97, 200, 520]), max_pos=s, ln_eps=rng.choice([1e-5, 1e-12]))
        out.append((cfg, rng.choice([B.ORDER_EARLY_BACKWARD, B.ORDER_GPIPE]),
                    rng.choice([0, 0, B.FLAG_RECOMPUTE, B.FLAG_ONE_STREAM])))
    return out


@pytest.mark.parametrize("seed,n,big", [(11, 24, False), (12, 16, True)])
def test_random_shapes_follow_the_oracle(seed, n, big):
    for i, (cfg, order, flags) in enumerate(_cases(seed, n, big)):
        print(f"case {i}: {cfg} order={order} flags={flags}", flush=True)
        theta, mbs = make_inputs(cfg, 1000 * seed + i, cfg.M)
        got = run_gpu(cfg, theta, mbs, cfg.M, cfg.K, order, flags=flags)
        st, ref = run_oracle(cfg, theta, mbs, cfg.M, cfg.K)
        compare(cfg, st, ref, got, 1e-4 if cfg.dtype == "f32" else 2e-2, cfg.M, mbs)
