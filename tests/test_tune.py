"""The tuning script: its statistics (CPU) and a short sweep on the GPU."""
import json

import pytest

from paper_2205_00618_amd import tune


def test_statistics_of_the_named_workloads():
    s = tune.sgemm_stats(4096, 4096, 4096)
    assert s.ops == 2.0 * 4096**3 and s.bytes == 4 * 4 * 4096**2 and s.intensity == 512.0
    c = tune.conv_stats(32, 56, 56, 64, 64, 3, 3, 1, 1)
    assert c.ops == 2.0 * 32 * 56 * 56 * 64 * 576
    assert c.bytes == 4.0 * (2 * 32 * 56 * 56 * 64 + 64 * 576)
    d = tune.dwconv_stats(1, 112, 112, 16, 3, 3, 2, 1)
    assert d.ops == 2.0 * 56 * 56 * 16 * 9 and d.bytes == 1004096.0
    assert tune.sgemm_stats(8, 8, 8, elem_in=1).bytes == 2 * 64 + 2 * 4 * 64


def test_staging_families():
    assert tune.staging_family("sgemm_128x128x16_w2x2") == "register-staged"
    assert tune.staging_family("sgemm_dma_128x128x16_w2x2_s2_c0") == "direct-to-LDS"
    assert tune.staging_family("sgemm_dma_edge_64x64x16_w2x1_s3") == "direct-to-LDS (ragged)"
    assert tune.staging_family("sgemm_rows_16x64x64_w4") == "global to registers"
    assert tune.staging_family("conv2d_dma_64x64x32_w2x2_s2") == "direct-to-LDS"
    assert tune.staging_family("dwconv_window_3x3_s1_v4") == "register window"
    assert tune.staging_family("dwconv_lds_5x5_s1_tp1") == "LDS-staged"
    assert tune.staging_family("dwconv_direct_vec4") == "direct"


def test_random_shapes_are_seeded_and_bounded():
    a, b2 = tune.random_shapes(7, 40), tune.random_shapes(7, 40)
    assert a == b2 and a != tune.random_shapes(8, 40) and len(a) == 40
    for M, N, K in a:
        assert 1 <= M <= 8192 and 1 <= N <= 8192 and 1 <= K <= 8192
        assert M * N * K <= 2.5e11 and M * N <= 6e7
    assert any(M % 4 for M, _, _ in tune.random_shapes(7, 200)), "some shapes have unaligned rows"
    assert tune.random_igemm_shapes(3, 30) == tune.random_igemm_shapes(3, 30)
    assert all(N % 4 == 0 for _, N, _ in tune.random_igemm_shapes(3, 100))
    skinny = tune.random_skinny_shapes(9, 40)
    assert skinny == tune.random_skinny_shapes(9, 40) and all(min(M, N) <= 32 and K % 4 == 0 for M, N, K in skinny)
    convs = tune.random_conv_shapes(5, 30)
    assert convs == tune.random_conv_shapes(5, 30) and all(len(c) == 9 and c[8] == c[5] // 2 for c in convs)


@pytest.mark.gpu
@pytest.mark.parametrize("argv", [["sgemm", "384", "256", "512"], ["conv", "1", "14", "14", "64", "64", "3", "3", "1", "1"],
                                  ["dwconv", "4", "28", "28", "16", "3", "3", "1", "1"], ["igemm", "512", "384", "1024"],
                                  ["sgemm", "256", "192", "2048", "--workspace"]])
def test_sweep_finds_a_configuration_no_slower_than_the_default(argv, capsys, monkeypatch):
    from paper_2205_00618_amd import binding as b
    print("case: tune", argv, flush=True)
    monkeypatch.setattr(tune.Sweep, "__init__", _short_sweep(tune.Sweep.__init__))
    assert tune.main(argv) == 0
    out = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert out["candidates"] >= 4 and out["best"]["us"] > 0 and out["arithmetic_intensity"] > 0
    # every candidate reproduced the bits of the library's own choice on small-integer operands
    assert out["verified"] and out["wrong"] == []
    # the overrides are switched off again
    assert b.set_tuning(-1, 0) == b.OK


def _short_sweep(init):
    def wrapped(self, *a, **kw):
        kw["min_ms"] = 2.0
        init(self, *a, **kw)
    return wrapped


@pytest.mark.gpu
def test_a_candidate_with_a_wrong_result_never_wins(monkeypatch):
    """The sweep's check, with the mistake planted on the host: a candidate whose exact run
    returns something else is marked wrong and left out of the ranking."""
    import torch
    from paper_2205_00618_amd import binding as b
    b.use_torch_stream()
    A, B = torch.ones(64, 64, device="cuda"), torch.ones(64, 64, device="cuda")
    C, Ci = torch.zeros(64, 64, device="cuda"), torch.zeros(64, 64, device="cuda")
    state = {"bad": False}

    def exact():
        Ci.zero_()
        b.sgemm_t(A, B, Ci)
        return Ci + 1 if state["bad"] else Ci

    sweep = tune.Sweep(tune.sgemm_stats(64, 64, 64), lambda: b.sgemm_t(A, B, C), lambda: None, torch, b,
                       min_ms=1.0, exact=exact)
    good = sweep.measure(tune.Candidate(1, "good", lambda: None))
    state["bad"] = True
    bad = sweep.measure(tune.Candidate(1, "bad", lambda: None))
    assert good.ok and not bad.ok
    bad.us = 0.0   # however fast
    assert sweep.best() is good


@pytest.mark.gpu
def test_the_oracle_agrees_with_what_the_sweep_accepts():
    """The sweep compares candidates with the library's own choice; here that reference itself is
    held against the CPU oracle on the same kind of small-integer operands."""
    import numpy as np
    import torch
    import oracle
    from paper_2205_00618_amd import binding as b
    b.use_torch_stream()
    b.set_tuning(-1, 0)
    torch.manual_seed(5)
    A, B = tune.small_integers(torch, (200, 300)), tune.small_integers(torch, (300, 130))
    C = torch.zeros(200, 130, device="cuda")
    b.sgemm_t(A, B, C)
    torch.cuda.synchronize()
    ref, _ = oracle.sgemm(A.cpu().numpy(), B.cpu().numpy(), np.zeros((200, 130), np.float32))
    assert np.array_equal(C.cpu().numpy().astype(np.float64), ref)


@pytest.mark.gpu
def test_built_in_choice_stays_close_to_the_best_forced_kernel(capsys):
    """On a handful of shapes the kernel and cut the library picks by itself must not be more
    than 10 % behind the best forced one (best of three timings each)."""
    shapes = [(1024, 1024, 1024), (1000, 1000, 1000), (4096, 4096, 256), (1536, 1536, 1536), (256, 256, 8192),
              (2000, 100, 1000)]
    rows = tune.choice_table(shapes, min_ms=5.0)
    print(capsys.readouterr().out, flush=True)
    for r in rows:
        assert r["ratio"] <= 1.10, r
