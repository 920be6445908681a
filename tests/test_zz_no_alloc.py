"""meft_route_static, the entry point for callers that cannot allocate: same results as meft_route, bit for bit
(it runs the same kernels on a fixed array inside the library instead of a caller's workspace), on two calls in a
row of which the second has the smaller input, and its size limit."""
import pytest

from paper_2406_04984_amd import synth

pytestmark = pytest.mark.gpu


def _route_both(cfg, bias=False):
    import torch
    from paper_2406_04984_amd import binding as B
    from paper_2406_04984_amd.harness import DeviceLayer
    t = synth.make_inputs(cfg)
    if bias:
        import numpy as np
        t.bias = np.linspace(-0.5, 0.5, cfg.n_blocks).astype(np.float32)
    la = DeviceLayer(t, B)
    la.route()                                   # meft_route: partial scores in the caller's workspace
    torch.cuda.synchronize()
    want_idx, want_score = la.block_idx.clone(), la.block_score.clone()
    la.block_idx.fill_(-1)
    la.block_score.fill_(float("nan"))
    B.meft_route_static(la.shape, la.h, la.Wg, la.bias, la.block_idx, la.block_score)
    torch.cuda.synchronize()
    assert torch.equal(la.block_idx, want_idx), cfg.name
    assert torch.equal(la.block_score, want_score), cfg.name
    return la


def test_two_calls_in_a_row_the_second_smaller():
    # bf16 on the matrix-core kernel with four partial score matrices (2.9 MB of the static array), then a
    # smaller fp32 problem whose single score matrix lands in the part the first call left behind
    _route_both(synth.small_case(T=3000, d=256, n_blocks=60, block_size=16, top_e=4, top_k=8, dtype="bf16", seed=1201))
    _route_both(synth.small_case(T=77, d=72, n_blocks=5, block_size=8, top_e=3, top_k=4, dtype="f32", seed=1202),
                bias=True)
    # and the larger one again after the smaller
    _route_both(synth.small_case(T=3000, d=256, n_blocks=60, block_size=16, top_e=4, top_k=8, dtype="bf16", seed=1203))


def test_headline_shape_fits_and_matches():
    cfg = synth.CONFIGS["small_bf16"]
    _route_both(cfg)


def test_beyond_the_limit_is_refused_before_anything_runs():
    import torch
    from paper_2406_04984_amd import binding as B
    # 16 * T * n_blocks = 16.8 MB > 16 MiB
    s = B.make_shape(4100, 64, 256, 16, 2, 8, "bf16")
    h = torch.zeros((4100, 64), dtype=torch.bfloat16, device="cuda")
    wg = torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda")
    bi = torch.full((4100, 2), -7, dtype=torch.int32, device="cuda")
    rc = B.meft_route_static(s, h, wg, None, bi, None, check=False)
    torch.cuda.synchronize()
    assert rc == B.MEFT_ERR_WORKSPACE
    assert bool((bi == -7).all())
    # the largest problem the array holds: 16 * 4096 * 256 bytes exactly
    s = B.make_shape(4096, 64, 256, 16, 2, 8, "bf16")
    assert B.meft_route_static(s, h[:4096], wg, None, bi[:4096], None, check=False) == B.MEFT_OK
    torch.cuda.synchronize()
    assert bool((bi[:4096] >= 0).all())
