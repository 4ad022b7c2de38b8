"""Random legal shapes through the public entry points against the fp64 oracle: plain and masked queries on every key
type, fp8 queries, weighted random selection.  The shapes are drawn from a seeded generator so that the row count,
batch size, k and row length fall on both sides of every switch between kernels (small-knowledge-base path, tile
heights, query blocks of 32 / 64 / 128 / 256, full-line and tiled kernels)."""
import numpy as np
import pytest
import torch

from oracle import compare, kb_oracle
from paper_2602_14293_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import kb_testlib

    return kb_testlib


def _case(rng):
    kind = str(rng.choice(["bf16", "bf16m", "f32", "fp8", "fp8q8", "draw", "drawm"]))
    N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 20000), rng.integers(20000, 120000), rng.integers(250000, 300000)]))
    Q = int(rng.choice([rng.integers(1, 33), rng.integers(33, 129), rng.integers(129, 257), rng.integers(257, 520)]))
    k = int(rng.choice([1, rng.integers(2, 33), rng.integers(33, 129)]))
    d = int(rng.choice([64, 128, 256, 320, 512, 768, 1024]))
    if kind == "f32":
        d = max(32, d // 2)
    return kind, N, Q, k, d, int(rng.integers(1, 1 << 30))


@pytest.mark.parametrize("seed", [11, 23, 47])
def test_random_shapes_agree_with_the_oracle(T, seed):
    rng = np.random.default_rng(seed)
    done = 0
    while done < 40:
        kind, N, Q, k, d, s = _case(rng)
        if N * Q * d > 3e9:                       # keeps the oracle's share of the test to seconds
            continue
        label = f"{kind} N={N} d={d} Q={Q} k={k} seed={s}"
        centers = max(1, min(64, N // 4))
        if kind in ("bf16", "draw"):
            w = W.clustered(seed=s, N=N, d=d, Q=Q, k=k, centers=centers)
        elif kind in ("bf16m", "drawm"):
            w = W.filtered(seed=s, N=N, d=d, Q=Q, k=k, centers=centers)
        elif kind == "f32":
            w = W.tiny(seed=s, N=N, d=d, Q=Q, k=k)
        else:
            w = W.compressed(seed=s, N=N, d=d, Q=Q, k=k, centers=centers, fp8_queries=(kind == "fp8q8"))
        if kind.startswith("draw"):
            gain = np.random.default_rng(s).uniform(0.25, 4.0, size=w.N).astype(np.float32)
            gain[::7] = 0.0
            kb = T.build_kb(w)
            qm = w.qmask.cuda() if w.qmask is not None else None
            gi, gk = kb.query_sampled(w.queries.cuda().contiguous(), w.k, torch.from_numpy(gain).cuda(), 0.05, s, qm)
            torch.cuda.synchronize()
            kb.close()
            keys = kb_oracle.selection_keys(T.oracle_scores(w), gain, 0.05, s, 0)
            tags = W.word_bits(w.tags) if w.qmask is not None else None
            qmb = W.word_bits(w.qmask) if w.qmask is not None else None
            rep, _ = compare.check(gi.cpu().numpy(), gk.cpu().numpy(), keys, w.k, 2e-4, tags=tags, qmask=qmb, label=label, tight_tau=2e-5)
            assert rep.max_score_err <= 2e-5, f"{label}: key error {rep.max_score_err:.2e}"
        else:
            T.run_and_check(w, use_mask=True, label=label)
        done += 1
