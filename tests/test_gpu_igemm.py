"""GPU parity (bit-exact) of igemm_s8s32 against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    yield
    b.set_tuning(-1, 0)


def run_igemm(A, B, C, lda=None, ldb=None, ldc=None, offset=0):
    M, K = A.shape
    N = B.shape[1]
    lda, ldb, ldc = lda or K, ldb or N, ldc or N

    def place(a, ld, fill):
        buf = np.full(a.shape[0] * ld + offset, fill, a.dtype)
        buf[offset:].reshape(a.shape[0], ld)[:, :a.shape[1]] = a
        return buf

    dA, dB, dC = dev(place(A, lda, 77)), dev(place(B, ldb, 77)), dev(place(C, ldc, 777))
    st = b.igemm_s8s32(M, N, K, dA.data_ptr() + offset, lda, dB.data_ptr() + offset, ldb,
                       dC.data_ptr() + 4 * offset, ldc)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    full = out[offset:].reshape(M, ldc)
    assert np.all(full[:, N:] == 777) and np.all(out[:offset] == 777), "wrote outside C"
    return full[:, :N].copy()


def check(shape, seed, c_zero=False, **kw):
    A, B, C = wl.igemm_inputs(seed, wl.GemmShape(*shape), c_zero=c_zero)
    got = run_igemm(A, B, C, **kw)
    ref = oracle.igemm_s8s32(A, B, C)
    assert np.array_equal(got, ref), f"{shape} {b.last_variant()}: {int((got != ref).sum())} mismatches"


def test_hand_sum_on_gpu():
    A = np.array([[-128, 127], [127, -128]], np.int8)
    B = np.array([[-128, 127], [-128, 127]], np.int8)
    got = run_igemm(A, B, np.zeros((2, 2), np.int32))
    assert np.array_equal(got, np.array([[128, -127], [128, -127]], np.int32))


def test_config_igemm_1024():
    seed, shape = wl.IGEMM_1024
    print("case: igemm 1024^3 seed", seed, flush=True)
    check((shape.M, shape.N, shape.K), seed, c_zero=True)
    print("   variant", b.last_variant(), flush=True)


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 64), (65, 63, 65), (130, 70, 200),
                                   (1, 300, 33), (300, 1, 33), (257, 255, 129), (128, 128, 4096)])
def test_ragged_shapes(shape):
    print("case: igemm", shape, flush=True)
    check(shape, sum(shape))


@pytest.mark.parametrize("split", [1, 2, 5])
def test_split_k_is_bit_exact(split):
    assert b.set_tuning(-1, split) == b.OK
    check((200, 136, 1000), 90 + split)


def test_large_tiles():
    check((2944, 2944, 192), 95)
    assert b.last_variant() == "igemm_128x128x64"
    check((2940, 2949, 200), 96)


@pytest.mark.parametrize("lda,ldb,ldc,offset", [(272, 144, 140, 0), (259, 139, 137, 0),
                                                (272, 144, 140, 1), (272, 144, 140, 16)])
def test_leading_dimensions_and_misaligned_bases(lda, ldb, ldc, offset):
    check((100, 136, 256), 97, lda=lda, ldb=ldb, ldc=ldc, offset=offset)


def test_all_minimum_values():
    A = np.full((64, 1024), -128, np.int8)
    B = np.full((1024, 64), -128, np.int8)
    got = run_igemm(A, B, np.zeros((64, 64), np.int32))
    assert np.all(got == 2**24)


def test_k_zero_leaves_c():
    C = np.arange(12, dtype=np.int32).reshape(3, 4)
    dC = dev(C)
    assert b.igemm_s8s32(3, 4, 0, 0, 1, 0, 4, dC.data_ptr(), 4) == b.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C)
