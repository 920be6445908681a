"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU): every entry point is run
once on a seeded case by a small C driver built together with oracle/meft_oracle.c; any report aborts the driver.
Its results must equal those of the ordinary build, which the pins check."""
import os
import subprocess

import numpy as np
import pytest

from oracle import oracle
from paper_2406_04984_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitize_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
                           os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
                           os.path.join(ROOT, "oracle", "meft_oracle.c"), "-lm"])
    return exe


@pytest.mark.parametrize("kw", [
    dict(T=37, d=24, n_blocks=5, block_size=12, top_e=2, top_k=7),
    dict(T=9, d=8, n_blocks=3, block_size=4, top_e=3, top_k=12),      # everything selected
    dict(T=5, d=16, n_blocks=1, block_size=40, top_e=1, top_k=1),     # one block, one neuron
])
def test_every_entry_point_under_asan_and_ubsan(driver, tmp_path, kw):
    cfg = synth.small_case(dtype="f32", seed=77, **kw)
    t = synth.make_inputs(cfg)
    T, d, B, N, e, k, C = cfg.T, cfg.d, cfg.n_blocks, cfg.N, cfg.top_e, cfg.top_k, cfg.C
    bias = np.linspace(-0.3, 0.3, B).astype(np.float32)
    rows = np.array(sorted({0, N - 1, N // 2}), np.int32)
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        np.array([T, d, B, cfg.block_size, e, k, rows.size], np.int32).tofile(f)
        for a in (t.h, t.Wg, bias, t.K, t.V, t.dOut):
            np.ascontiguousarray(a, np.float32).tofile(f)
        rows.tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    p = subprocess.run([driver, fin, fout], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       timeout=300)
    assert p.returncode == 0, p.stdout[-4000:]
    assert "runtime error" not in p.stdout and "AddressSanitizer" not in p.stdout, p.stdout[-4000:]

    # the same calls through the ordinary build
    r = oracle.route(t.h, t.Wg, e, bias)
    fw = oracle.forward(t.h, t.K, t.V, r.block_idx, cfg.block_size, k, want_candidates=True)
    bw = oracle.backward(t.h, t.K, t.V, fw.idx, fw.score, t.dOut, cfg.block_size)
    bw_rows = oracle.backward(t.h, t.K, t.V, fw.idx, fw.score, t.dOut, cfg.block_size, rows=rows, want_dh=False)
    applied = oracle.apply_selection(t.h, t.K, t.V, fw.idx, cfg.block_size)
    S = bw.touched
    u_out = oracle.union_forward(t.h, t.K, t.V, S)
    u_dh, u_dK, u_dV = oracle.union_backward(t.h, t.K, t.V, S, t.dOut)
    w, m, v = oracle.adam_rows(t.K.astype(np.float64), bw.dK, 0.1 * bw.dV, 0.01 * bw.dV * bw.dV, S, step=3, lr=1e-3)

    raw = np.fromfile(fout, np.uint8)
    pos = 0

    def take(dtype, *shape):
        nonlocal pos
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        a = raw[pos:pos + n].view(dtype).reshape(shape)
        pos += n
        return a

    def same(a, b):
        assert np.array_equal(np.asarray(a), np.asarray(b))

    same(take(np.int32, T, e), r.block_idx); same(take(np.float64, T, e), r.block_score); same(take(np.float64, T, B), r.p)
    same(take(np.float64, T, d), fw.out); same(take(np.int32, T, k), fw.idx); same(take(np.float64, T, k), fw.score)
    same(take(np.float64, T), fw.next_score); same(take(np.int32, T, C), fw.cand_id)
    same(take(np.float64, T, C), fw.cand_score)
    same(take(np.float64, T, d), bw.dh); same(take(np.float64, N, d), bw.dK); same(take(np.float64, N, d), bw.dV)
    nt = int(take(np.int32, 1)[0])
    assert nt == S.size
    same(take(np.int32, nt), S)
    same(take(np.float64, rows.size, d), bw_rows.dK); same(take(np.float64, rows.size, d), bw_rows.dV)
    same(take(np.float64, T, d), applied)
    same(take(np.float64, T, d), u_out); same(take(np.float64, T, d), u_dh)
    same(take(np.float64, nt, d), u_dK); same(take(np.float64, nt, d), u_dV)
    same(take(np.float64, N, d), w); same(take(np.float64, N, d), m); same(take(np.float64, N, d), v)
    rc, refused = take(np.int32, 2)
    assert rc == 0 and refused == 6
    assert pos == raw.size
