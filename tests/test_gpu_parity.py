"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle (pytest -m gpu)."""
import numpy as np
import pytest

from paper_2406_04984_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import parity
    return parity


def _case(P, **kw):
    cfg = synth.small_case(**kw)
    rep = P.run_and_compare(cfg)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    return rep


def test_config_tiny_f32(P):
    rep = P.run_and_compare(synth.CONFIGS["tiny_f32"])
    print(rep.summary(), flush=True)
    rep.assert_ok()
    assert rep.idx_band_tokens == 0 and rep.block_band_tokens == 0


def test_config_small_bf16(P):
    rep = P.run_and_compare(synth.CONFIGS["small_bf16"])
    print(rep.summary(), flush=True)
    rep.assert_ok()


def _full_size(P, name, n_rows=384):
    """The benchmark's launch configuration at full size: every token's selections, and out and dh row by row,
    against the oracle; dK / dV on a stratified sample of neuron rows that the oracle computes one by one: of
    every block the first and last neuron and the rows on both sides of every 128-row tile boundary, plus
    seeded random rows."""
    cfg = synth.CONFIGS[name]
    rows = P.stratified_rows(cfg, n_rows)
    rep = P.run_and_compare(cfg, rows=rows)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    return rep


@pytest.mark.timeout(900)
def test_config_llama7b_bf16_full_size(P):
    _full_size(P, "llama7b_bf16")


@pytest.mark.timeout(900)
def test_config_wide_bf16_full_size(P):
    _full_size(P, "wide_bf16")


@pytest.mark.timeout(900)
def test_config_llama7b_hostkv_bf16_full_size(P):
    """Keys and values (131072 x 4096, 128 blocks) in pinned host memory, gradients written back to pinned host
    memory: the staged block copies, the kept copies in the backward and the row write-back at full size."""
    _full_size(P, "llama7b_hostkv_bf16")


def test_eight_blocks_per_token_on_the_matrix_core_path(P):
    """top_e = 8: a token's output and input gradient are sums of eight per-block partial rows, each rounded to
    bf16 before the fp32 sum (the rounding points the header states); judged row by row like everything else."""
    _case(P, T=400, d=256, n_blocks=12, block_size=128, top_e=8, top_k=200, dtype="bf16", seed=707)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_shapes(P, dtype):
    # token count, block size, hidden size and candidate count all off the tile sizes
    _case(P, T=77, d=72, n_blocks=5, block_size=40, top_e=3, top_k=17, dtype=dtype, seed=101)
    _case(P, T=300, d=200, n_blocks=7, block_size=150, top_e=2, top_k=33, dtype=dtype, seed=102)
    _case(P, T=130, d=2056, n_blocks=3, block_size=24, top_e=2, top_k=9, dtype=dtype, seed=103)


def test_ragged_shapes_on_the_matrix_core_path(P):
    """bf16 shapes that take the block-dense path (hidden size a multiple of 64) with token groups, block
    sizes and hidden sizes off the 128 x 256 x 64 tile, an empty block, and one block taking every token."""
    _case(P, T=333, d=192, n_blocks=5, block_size=72, top_e=2, top_k=19, dtype="bf16", seed=701)
    _case(P, T=130, d=320, n_blocks=3, block_size=300, top_e=3, top_k=100, dtype="bf16", seed=702)
    _case(P, T=700, d=64, n_blocks=20, block_size=16, top_e=5, top_k=40, dtype="bf16", seed=703)
    _case(P, T=257, d=512, n_blocks=2, block_size=520, top_e=1, top_k=65, dtype="bf16", seed=704)
    _case(P, T=90, d=64, n_blocks=4, block_size=30, top_e=2, top_k=12, dtype="bf16", seed=706)
    cfg = synth.small_case(T=200, d=128, n_blocks=6, block_size=64, top_e=2, top_k=24, dtype="bf16", seed=705)
    t = synth.make_inputs(cfg)
    t.bias = np.array([0, 50, -50, 0, 0, 0], np.float32)     # block 1 takes every token, block 2 none
    from oracle import oracle
    g = P.run_gpu(t)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    b = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, cfg.block_size)
    rep = P.compare(t, g, r, f, b)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    assert (g["block_idx"][:, 0] == 1).all() and (g["block_idx"] != 2).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_selections(P, dtype):
    _case(P, T=33, d=64, n_blocks=4, block_size=16, top_e=4, top_k=64, dtype=dtype, seed=201)   # dense adapter
    _case(P, T=33, d=64, n_blocks=1, block_size=96, top_e=1, top_k=10, dtype=dtype, seed=202)   # one expert
    _case(P, T=33, d=64, n_blocks=6, block_size=16, top_e=2, top_k=32, dtype=dtype, seed=203)   # k = C
    _case(P, T=33, d=64, n_blocks=6, block_size=16, top_e=1, top_k=1, dtype=dtype, seed=204)    # one neuron
    _case(P, T=1, d=64, n_blocks=6, block_size=16, top_e=2, top_k=5, dtype=dtype, seed=205)     # one token
    _case(P, T=40, d=8, n_blocks=48, block_size=1, top_e=6, top_k=6, dtype=dtype, seed=206)     # one neuron per expert


def test_matrix_core_scores_on_the_gather_path(P):
    """bf16 shapes too sparse for the block-dense kernels (64 top_k < candidates) still score on the matrix-core
    kernel when the hidden size is a multiple of 64 and the groups are large; everything after the scores is the
    per-pair path.  One and three groups: fewer groups than XCDs, so every XCD takes every eighth tile."""
    _case(P, T=600, d=128, n_blocks=1, block_size=9000, top_e=1, top_k=20, dtype="bf16", seed=221)
    _case(P, T=700, d=192, n_blocks=3, block_size=3000, top_e=2, top_k=33, dtype="bf16", seed=222)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_selection_larger_than_one_output_staging_round(P, dtype):
    """top_k beyond the 1024 selections that the selection kernel stages per round, candidate counts on and off the
    kernel's 256 x keys-per-thread grid."""
    _case(P, T=21, d=64, n_blocks=4, block_size=1024, top_e=2, top_k=1500, dtype=dtype, seed=211)   # C = 2048 = 256 * 8
    _case(P, T=21, d=64, n_blocks=5, block_size=700, top_e=3, top_k=2049, dtype=dtype, seed=212)    # C = 2100


def test_tokens_whose_scores_are_all_equal(P):
    """Zero rows of h give all-zero scores: every digit of every key is the same (the histogram passes see one bin),
    the first top_k candidates are selected and contribute nothing."""
    cfg = synth.small_case(T=48, d=64, n_blocks=6, block_size=64, top_e=2, top_k=30, dtype="bf16", seed=213)
    t = synth.make_inputs(cfg)
    t.h[::3] = 0.0
    from oracle import oracle
    g = P.run_gpu(t)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    b = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, cfg.block_size)
    rep = P.compare(t, g, r, f, b)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    assert (g["idx"][::3] == np.sort(f.idx, 1)[::3]).all()
    assert (g["act"][::3] == 0).all() and (g["out"][::3] == 0).all()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 72)])
def test_keys_and_values_in_pinned_host_memory(P, dtype, d):
    """MEFT_FLAG_HOST_KV: K, V are read from, and the touched rows of dK, dV written to, pinned host memory.
    Same kernels as the device-resident path, so the results must be bit-identical to it; block 3 is never
    routed to, so its rows are neither fetched nor written."""
    cfg = synth.small_case(T=150, d=d, n_blocks=6, block_size=32, top_e=2, top_k=12, dtype=dtype, seed=801)
    t = synth.make_inputs(cfg)
    t.bias = np.array([0, 0, 0, -100, 0, 0], np.float32)
    ref = P.run_gpu(t)
    th = synth.Tensors(cfg.replace(host_kv=True), t.h, t.Wg, t.K, t.V, t.dOut, t.bias, t.outlier_channels)
    got = P.run_gpu(th)
    for n in ("block_idx", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched"):
        assert (ref[n] == got[n]).all(), n
    assert not ((got["touched"] >= 96) & (got["touched"] < 128)).any()
    # MEFT_FLAG_KEEP_STAGED: the backward reuses the blocks the forward staged instead of fetching them again
    tk = synth.Tensors(cfg.replace(host_kv=True, keep_staged=True), t.h, t.Wg, t.K, t.V, t.dOut, t.bias,
                       t.outlier_channels)
    kept = P.run_gpu(tk)
    for n in ("block_idx", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched"):
        assert (ref[n] == kept[n]).all(), n
    from oracle import oracle
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    b = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, cfg.block_size)
    rep = P.compare(th, got, r, f, b)
    print(rep.summary(), flush=True)
    rep.assert_ok()


def test_dense_case_matches_numpy_dense_adapter(P):
    """top_e = n_blocks, top_k = N: the GPU result is the dense parallel adapter (Section 2)."""
    from oracle import dense_ref
    cfg = synth.small_case(T=50, d=64, n_blocks=4, block_size=32, top_e=4, top_k=128, dtype="f32", seed=301)
    t = synth.make_inputs(cfg)
    g = P.run_gpu(t)
    dh, dK, dV = dense_ref.dense_adapter_grads(t.h, t.K, t.V, t.dOut)
    assert P.rel_l2(g["out"], dense_ref.dense_adapter(t.h, t.K, t.V)) < 1e-4
    assert P.rel_l2(g["dh"], dh) < 1e-4 and P.rel_l2(g["dK"], dK) < 1e-4 and P.rel_l2(g["dV"], dV) < 1e-4


def test_empty_batch(P):
    import torch
    from paper_2406_04984_amd import binding as B
    s = B.make_shape(0, 64, 4, 16, 2, 8, "bf16")
    ws = torch.empty((B.meft_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
    z = torch.zeros((16,), dtype=torch.int32, device="cuda")
    w = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    nt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.meft_route(s, w, w, None, z, None, ws)
    B.meft_sparse_fwd(s, w, w, w, z, w, z, z.float(), ws)
    B.meft_sparse_bwd(s, w, w, w, z, z.float(), w, None, w, w, z, nt, ws)
    torch.cuda.synchronize()
    assert int(nt.item()) == 0


def test_exact_ties_go_to_the_lower_index(P):
    """Duplicated router rows and duplicated keys give exactly equal scores on both sides."""
    cfg = synth.small_case(T=64, d=64, n_blocks=8, block_size=32, top_e=3, top_k=20, dtype="bf16", seed=401)
    t = synth.make_inputs(cfg)
    t.Wg[5] = t.Wg[2]
    t.Wg[7] = t.Wg[2]
    t.K[1::2] = t.K[0::2]          # every odd neuron duplicates its even neighbour
    t.K[40:48] = 0.0               # a run of exact zeros (+0 and -0 both appear through the products)
    from oracle import oracle
    g = P.run_gpu(t)
    r = oracle.route(t.h, t.Wg, cfg.top_e, t.bias)
    f = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k, want_candidates=True)
    b = oracle.backward(t.h, t.K, t.V, f.idx, f.score, t.dOut, cfg.block_size)
    rep = P.compare(t, g, r, f, b)
    print(rep.summary(), flush=True)
    rep.assert_ok()
    # equal scores are exactly equal in both precisions here, so no tie band is needed
    assert (np.sort(g["block_idx"], 1) == np.sort(r.block_idx, 1)).all()
    assert (g["idx"] == np.sort(f.idx, 1)).all()


def test_backward_accepts_any_order_inside_a_token_and_is_deterministic(P):
    import torch
    cfg = synth.small_case(T=200, d=128, n_blocks=8, block_size=64, top_e=2, top_k=24, dtype="bf16", seed=501)
    t = synth.make_inputs(cfg)
    L = P.DeviceLayer(t)
    L.fill_grad_sentinel()
    L.step()
    a = L.results()
    rng = np.random.default_rng(5)
    perm = np.stack([rng.permutation(cfg.top_k) for _ in range(cfg.T)])
    pt = torch.from_numpy(perm).cuda()
    L.idx.copy_(torch.gather(L.idx, 1, pt))
    L.act.copy_(torch.gather(L.act, 1, pt))
    L.fill_grad_sentinel()
    L.bwd()
    b = L.results()
    # dK, dV sum pairs in token order whatever the order inside a token: bit-identical
    assert (a["dK_bits"] == b["dK_bits"]).all() and (a["dV_bits"] == b["dV_bits"]).all()
    assert (a["touched"] == b["touched"]).all()
    assert P.rel_l2(b["dh"], a["dh"]) < 2e-2
    # same inputs again: every output bit-identical
    L.fill_grad_sentinel()
    L.bwd()
    c = L.results()
    for n in ("dK_bits", "dV_bits", "dh", "touched"):
        assert (b[n] == c[n]).all(), n


def test_two_full_runs_are_bit_identical(P):
    cfg = synth.small_case(T=257, d=256, n_blocks=8, block_size=128, top_e=3, top_k=40, dtype="bf16", seed=601)
    t = synth.make_inputs(cfg)
    a, b = P.run_gpu(t), P.run_gpu(t)
    for n in ("block_idx", "block_score", "idx", "act", "out", "dh", "dK_bits", "dV_bits", "touched"):
        assert (a[n] == b[n]).all(), n
