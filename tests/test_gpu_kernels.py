"""Kernel-level GPU checks (single GEMM / attention launches) against plain fp64 numpy definitions.
These go through the kernel hooks of the library, not the stage ABI; the stage-level parity tests are
in test_gpu_stage.py."""
import ctypes as C
import math

import numpy as np
import pytest
import torch
from scipy.special import erf

import swarm_synth as synth

pytestmark = pytest.mark.gpu


def _lib():
    import paper_2301_11913_amd as sw
    lib = sw.load_library()
    lib.swarm_kernel_gemm.restype = C.c_int
    lib.swarm_kernel_gemm.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_void_p]
    return lib


def _bf(a):
    return torch.from_numpy(a).to(torch.bfloat16)


def _gelu(u):
    return 0.5 * u * (1 + erf(u / math.sqrt(2)))


def _gelu_grad(u):
    return 0.5 * (1 + erf(u / math.sqrt(2))) + u * np.exp(-0.5 * u * u) / math.sqrt(2 * math.pi)


def gemm_case(M, N, K, a_t, b_t, epi, seed=0):
    lib = _lib()
    A = _bf(synth.normal(seed, "A", (K, M) if a_t else (M, K)))
    B = _bf(synth.normal(seed, "B", (K, N) if b_t else (N, K)))
    bias = _bf(synth.normal(seed, "bias", (N,)))
    aux = _bf(synth.normal(seed, "aux", (M, N)))
    A64 = A.double().numpy(); B64 = B.double().numpy()
    ref = (A64.T if a_t else A64) @ (B64 if b_t else B64.T)
    Ad, Bd, bd, xd = A.cuda(), B.cuda(), bias.cuda(), aux.cuda()
    C2 = None
    if epi == 5:
        Cd = _bf(synth.normal(seed, "C0", (M, N))).float().cuda()
        ref = ref + Cd.double().cpu().numpy()
    else:
        Cd = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
        if epi == 1:
            ref = ref + bias.double().numpy()
        elif epi == 2:
            ref = ref + bias.double().numpy() + aux.double().numpy()
        elif epi == 3:
            C2 = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
            u = ref + bias.double().numpy()
            ref = _gelu(u)
        elif epi == 4:
            ref = ref * _gelu_grad(aux.double().numpy())
    st = lib.swarm_kernel_gemm(1, M, N, K, Ad.data_ptr(), A.shape[1], int(a_t), Bd.data_ptr(), B.shape[1], int(b_t),
                               Cd.data_ptr(), N, epi, bd.data_ptr(), xd.data_ptr(), N,
                               C2.data_ptr() if C2 is not None else None, N, None)
    assert st == 0
    torch.cuda.synchronize()
    got = Cd.double().cpu().numpy()
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    assert err < (1e-5 if epi == 5 else 6e-3), err
    if C2 is not None:
        e2 = np.max(np.abs(C2.double().cpu().numpy() - u)) / np.max(np.abs(u))
        assert e2 < 6e-3, e2


LAYOUTS = [(False, False), (False, True), (True, True)]


@pytest.mark.parametrize("a_t,b_t", LAYOUTS)
@pytest.mark.parametrize("shape", [(256, 256, 64), (128, 128, 128), (512, 768, 256), (300, 192, 320),
                                   (37, 64, 64), (1000, 1088, 200), (4096, 4096, 512), (2048, 4096 + 64, 256 + 64)])
def test_gemm_layouts(a_t, b_t, shape):
    M, N, K = shape
    if a_t and M % 8:
        M = (M + 7) // 8 * 8          # a transposed operand's row length is a feature dimension
    gemm_case(M, N, K, a_t, b_t, 5 if a_t else 0, seed=M + N + K)


@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("shape", [(384, 256, 128), (4096, 4096, 128), (77, 192, 64)])
def test_gemm_epilogues(epi, shape):
    M, N, K = shape
    gemm_case(M, N, K, False, epi == 4, epi, seed=epi)
