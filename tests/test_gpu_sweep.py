"""Seeded sweep of small shapes through both formulations (per-pair gather: fp32 and sparse bf16 shapes; block-dense
matrix-core: the other bf16 shapes) against the oracle: hidden sizes, block sizes and counts, top_e, top_k, token
counts from 1 to 1500, balanced and Zipf-biased routing (so that groups of every size occur, the ones the
contractions leave to the per-pair kernels included), with the forward's tables reused by the backward and rebuilt.
Same comparison rules as every other parity test."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth

pytestmark = pytest.mark.gpu


def _shapes(seed, n):
    rng = np.random.default_rng(seed)
    for it in range(n):
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        d = int(rng.choice([64, 128, 192, 256, 320, 512, 1024])) if dtype == "bf16" else int(rng.choice([8, 24, 72, 128, 200]))
        bs = int(rng.choice([16, 24, 40, 64, 72, 100, 128, 200, 256, 300, 512]))
        nb = int(rng.integers(1, 40))
        e = int(rng.integers(1, min(nb, 6) + 1))
        C = e * bs
        k = min(C, int(rng.integers(max(1, C // 64), max(2, min(C, 200)) + 1)))
        T = int(rng.choice([1, 3, 17, 64, 130, 257, 600, 1500]))
        yield synth.small_case(T=T, d=d, n_blocks=nb, block_size=bs, top_e=e, top_k=k, dtype=dtype, seed=2000 + it,
                               zipf_s=float(rng.choice([0.0, 0.0, 1.0, 2.0])), reuse_fwd=bool(rng.random() < 0.5))


@pytest.mark.parametrize("seed", [1, 2])
def test_random_small_shapes(seed):
    from tests import parity as P
    failures = []
    for cfg in _shapes(seed, 40):
        rep = P.run_and_compare(cfg)
        try:
            rep.assert_ok()
        except AssertionError as ex:
            failures.append(f"{cfg.name} zipf={cfg.zipf_s} reuse={cfg.reuse_fwd}: {str(ex)[:300]}")
    assert not failures, "\n".join(failures)
