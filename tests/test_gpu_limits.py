"""The documented limits of the build, exercised at their maxima (include/meft.h): hidden size 16384 on both
formulations, 16384 blocks, 4194304 candidates per token.  Same parity rules as everywhere else."""
import pytest

from paper_2406_04984_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    from tests import parity
    return parity


def _case(P, **kw):
    cfg = synth.small_case(**kw)
    rep = P.run_and_compare(cfg)
    print(rep.summary(), flush=True)
    rep.assert_ok()


def test_largest_hidden_size_on_the_matrix_core_path(P):
    _case(P, T=130, d=16384, n_blocks=4, block_size=64, top_e=2, top_k=16, dtype="bf16", seed=1001)


def test_largest_hidden_size_on_the_gather_path(P):
    _case(P, T=40, d=16384, n_blocks=4, block_size=64, top_e=2, top_k=16, dtype="f32", seed=1002)


def test_largest_number_of_blocks(P):
    _case(P, T=50, d=64, n_blocks=16384, block_size=2, top_e=3, top_k=4, dtype="f32", seed=1003)


@pytest.mark.timeout(600)
def test_largest_candidate_set(P):
    # two tokens over one block of 4194304 neurons
    _case(P, T=2, d=8, n_blocks=1, block_size=4194304, top_e=1, top_k=100, dtype="f32", seed=1004)


def test_dispatch_at_the_three_pass_limit_of_blocks(P):
    # 1024 blocks: the per-wave block counters of the three-pass dispatch fill 64 KB of LDS; several chunks of entries
    _case(P, T=700, d=64, n_blocks=1024, block_size=16, top_e=3, top_k=8, dtype="bf16", seed=1005)


def test_matrix_core_path_beyond_the_three_pass_dispatch(P):
    # more than 1024 blocks: the per-block dispatch kernels and the round-robin tile schedule, on the matrix-core path
    _case(P, T=300, d=64, n_blocks=1100, block_size=16, top_e=3, top_k=8, dtype="bf16", seed=1006)
