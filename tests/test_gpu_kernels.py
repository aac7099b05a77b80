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
    lib = sw.load_hooks_library()
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
                                   (37, 64, 64), (1000, 1088, 200), (4096, 4096, 512), (2048, 4096 + 64, 256 + 64),
                                   # whole tiles but K no multiple of 64: the register-staged kernels (128 x 128
                                   # and, from 160 big tiles on, 256 x 256), and a ragged M there
                                   (256, 384, 96), (4096, 2560, 96), (4104, 2560, 96),
                                   (40, 24, 20)])         # K no multiple of 8: the scalar kernel
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


# ------------------------------------------------------------------ split-K
def _splitk_call(lib, M, N, K, Ad, lda, Bd, ldb, b_t, Cd, epi, bd, xd, scales, ws):
    lib.swarm_kernel_gemm_ws.restype = C.c_int
    lib.swarm_kernel_gemm_ws.argtypes = [C.c_int] * 3 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                        C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    st = lib.swarm_kernel_gemm_ws(M, N, K, Ad.data_ptr(), lda, 0, Bd.data_ptr(), ldb, int(b_t), Cd.data_ptr(), N, epi,
                                  bd.data_ptr(), xd.data_ptr(), N, scales.data_ptr() if scales is not None else None,
                                  ws.data_ptr() if ws is not None else None, ws.numel() if ws is not None else 0, None)
    assert st == 0
    torch.cuda.synchronize()


# (M, N, K, parts the kernel takes): one tile cut in four, 16 tiles cut in two (K / 4 would be below 4096),
# 128 tiles cut in two, and a product that is not cut (K too short) although scratch is offered
@pytest.mark.parametrize("shape", [(256, 256, 16384), (512, 2048, 8192), (2048, 4096, 8192), (256, 512, 4096)])
@pytest.mark.parametrize("b_t", [False, True])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_gemm_splitk(shape, b_t, epi):
    M, N, K = shape
    lib = _lib()
    lib.swarm_kernel_gemm_splitk_floats.restype = C.c_size_t
    nfl = lib.swarm_kernel_gemm_splitk_floats(M, N)
    assert nfl == (4 if (M // 256) * (N // 256) <= 64 else 2) * M * N
    seed = M + N + K + epi
    A = _bf(synth.normal(seed, "A", (M, K)))
    B = _bf(synth.normal(seed, "B", (K, N) if b_t else (N, K)))
    bias = _bf(synth.normal(seed, "bias", (N,)))
    aux = _bf(synth.normal(seed, "aux", (M, N)))
    ref = A.double().numpy() @ (B.double().numpy() if b_t else B.double().numpy().T)
    if epi >= 1:
        ref = ref + bias.double().numpy()
    if epi == 2:
        ref = ref + aux.double().numpy()
    Ad, Bd, bd, xd = A.cuda(), B.cuda(), bias.cuda(), aux.cuda()
    ws = torch.full((nfl,), float("nan"), dtype=torch.float32, device="cuda")
    C1 = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
    _splitk_call(lib, M, N, K, Ad, K, Bd, B.shape[1], b_t, C1, epi, bd, xd, None, ws)
    got = C1.double().cpu().numpy()
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    assert err < 6e-3, err
    cut = K // 2 >= 4096
    assert bool(torch.isnan(ws).all()) == (not cut)            # the scratch is used exactly when K is long enough
    # the one-kernel product of the same operands: equal up to the summation order of the fp32 partial sums, i.e.
    # at most one bf16 unit (2^-7 of the element) apart after rounding
    C0 = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
    _splitk_call(lib, M, N, K, Ad, K, Bd, B.shape[1], b_t, C0, epi, bd, xd, None, None)
    d = np.max(np.abs(C0.double().cpu().numpy() - got)) / np.max(np.abs(ref))
    assert d <= 2.0 ** -7 and (cut or d == 0.0), d


@pytest.mark.parametrize("epi,b_t", [(0, False), (0, True), (1, False), (2, False), (3, False), (4, True)])
def test_gemm_ragged_last_round(epi, b_t):
    """384 tiles of 256 x 256 (one and a half rounds of the 256 compute units): the columns of the whole round and
    the remaining columns run as two products; every output column must come out as from one.  Epilogues with the
    layouts the stage uses them with."""
    gemm_case(2048, 12288, 256, False, b_t, epi, seed=40 + epi)


@pytest.mark.parametrize("epi,b_t", [(0, False), (0, True), (1, False), (2, False), (3, False), (4, True)])
@pytest.mark.parametrize("shape", [(2048, 4096, 64), (2048, 4096, 448), (1536, 4096, 256), (1792, 4224, 128)])
def test_gemm_256x128_tiles(shape, epi, b_t):
    """192 .. 256 tiles of 256 x 128 (a 2048-row microbatch times a 4096-wide weight): one round of those instead
    of two rounds of 128 x 128.  One, two, four and seven 64-deep slices; a column count that is no multiple of 256."""
    M, N, K = shape
    gemm_case(M, N, K, False, b_t, epi, seed=60 + epi)


@pytest.mark.parametrize("epi,b_t", [(0, False), (0, True), (1, False), (2, False), (3, False), (4, True)])
def test_gemm_streaming_outputs(epi, b_t):
    """Outputs of 64 MB and more are written, and their residual / pre-activation rows read, with non-temporal
    accesses (another copy of the epilogue code): 8192 x 4096 in bf16 is 64 MB."""
    gemm_case(8192, 4096, 128, False, b_t, epi, seed=70 + epi)


@pytest.mark.parametrize("epi", [0, 1, 2, 3, 6])
@pytest.mark.parametrize("shape", [(4096, 4096, 192), (8192, 4096, 128), (2560, 4096, 64)])
def test_gemm_four_wavefront_kernel_same_bits(epi, shape):
    """Forward products on 256 x 256 tiles run on four wavefronts of 128 x 128 (accumulators in place, epilogue on
    the accumulator layout); the instrumented library can send them to the eight-wavefront kernel instead.  Both
    accumulate in the same order and round once, so every output (C, the kept pre-activations, int8 codes and
    scales) has to agree bit for bit; 160, 256 and 512 tiles, cached and streaming stores, one to three slices."""
    M, N, K = shape
    lib = _lib()
    lib.swarm_kernel_gemm_ws.restype = C.c_int
    lib.swarm_kernel_gemm_ws.argtypes = [C.c_int] * 3 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                        C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    A = _bf(synth.normal(90 + epi, "A", (M, K))).cuda(); B = _bf(synth.normal(90 + epi, "B", (N, K))).cuda()
    bias = _bf(synth.normal(90 + epi, "bias", (N,))).cuda(); aux = _bf(synth.normal(90 + epi, "aux", (M, N))).cuda()
    outs = []
    for four in (1, 0):
        lib.swarm_kernel_gemm_four_waves(four)
        try:
            if epi == 6:
                Cd = torch.zeros((M, N), dtype=torch.int8, device="cuda")
                sc = torch.zeros(M * N // 64, dtype=torch.float32, device="cuda")
                st = lib.swarm_kernel_gemm_ws(M, N, K, A.data_ptr(), K, 0, B.data_ptr(), K, 0, Cd.data_ptr(), N, 6,
                                              bias.data_ptr(), aux.data_ptr(), N, sc.data_ptr(), None, 0, None)
                assert st == 0
                outs.append((Cd, sc.view(torch.int32)))
            else:
                res = []
                for keep_u in ((True, False) if epi == 3 else (False,)):
                    Cd = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
                    C2 = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda") if keep_u else None
                    st = lib.swarm_kernel_gemm(1, M, N, K, A.data_ptr(), K, 0, B.data_ptr(), K, 0, Cd.data_ptr(), N, epi,
                                               bias.data_ptr(), aux.data_ptr(), N,
                                               C2.data_ptr() if keep_u else None, N, None)
                    assert st == 0
                    res += [Cd.view(torch.int16)] + ([C2.view(torch.int16)] if keep_u else [])
                outs.append(tuple(res))
        finally:
            lib.swarm_kernel_gemm_four_waves(1)
    torch.cuda.synchronize()
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    if epi == 3:      # with and without the kept pre-activations: the same GeLU values
        assert torch.equal(outs[0][0], outs[0][2])


def test_gemm_splitk_encode_equals_encode_of_stored():
    """EPI 6 (bias + residual, int8-encoded) through the split path: codes and scales are those of the stand-alone
    codec applied to what the bias + residual epilogue stores (same scratch, same summation order)."""
    import paper_2301_11913_amd as sw
    M, N, K = 512, 1024, 8192
    lib = _lib()
    A = _bf(synth.normal(3, "A", (M, K))); B = _bf(synth.normal(3, "B", (N, K)))
    bias = _bf(synth.normal(3, "bias", (N,))); aux = _bf(synth.normal(3, "aux", (M, N)))
    Ad, Bd, bd, xd = A.cuda(), B.cuda(), bias.cuda(), aux.cuda()
    lib.swarm_kernel_gemm_splitk_floats.restype = C.c_size_t
    ws = torch.empty(lib.swarm_kernel_gemm_splitk_floats(M, N), dtype=torch.float32, device="cuda")
    Cb = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    _splitk_call(lib, M, N, K, Ad, K, Bd, K, False, Cb, 2, bd, xd, None, ws)
    codes = torch.empty((M, N), dtype=torch.int8, device="cuda")
    scales = torch.empty(M * N // 64, dtype=torch.float32, device="cuda")
    _splitk_call(lib, M, N, K, Ad, K, Bd, K, False, codes, 6, bd, xd, scales, ws)
    c2 = torch.empty(M * N, dtype=torch.int8, device="cuda"); s2 = torch.empty_like(scales)
    sw.swarm_codec_encode(Cb.reshape(-1), c2, s2)
    torch.cuda.synchronize()
    assert torch.equal(codes.reshape(-1), c2) and torch.equal(scales.view(torch.int32), s2.view(torch.int32))


# ------------------------------------------------------------------ attention
def _attn_lib():
    lib = _lib()
    lib.swarm_kernel_attention_fwd.restype = C.c_int
    lib.swarm_kernel_attention_fwd.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p]
    lib.swarm_kernel_attention_bwd.restype = C.c_int
    lib.swarm_kernel_attention_bwd.argtypes = [C.c_int] + [C.c_void_p] * 6 + [C.c_int] * 4 + [C.c_void_p]
    return lib


def _attn_ref(qkv, dout, B, S, H, dh):
    """fp64 definition: per (b,h) causal softmax(q k^T / sqrt(dh)) v and its gradient."""
    d = H * dh
    x = qkv.reshape(B, S, 3, H, dh).transpose(2, 0, 3, 1, 4)       # [3,B,H,S,dh]
    q, k, v = x[0], x[1], x[2]
    s = q @ k.transpose(0, 1, 3, 2) / math.sqrt(dh)
    mask = np.tril(np.ones((S, S), dtype=bool))
    s = np.where(mask, s, -np.inf)
    mx = s.max(-1, keepdims=True)
    e = np.exp(s - mx)
    den = e.sum(-1, keepdims=True)
    p = e / den
    o = p @ v
    lse = (mx + np.log(den))[..., 0]
    do = dout.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (p * dp).sum(-1, keepdims=True))
    dq = ds @ k / math.sqrt(dh)
    dk = ds.transpose(0, 1, 3, 2) @ q / math.sqrt(dh)
    back = lambda t: t.transpose(0, 2, 1, 3).reshape(B, S, d)
    return back(o), lse, np.concatenate([back(dq), back(dk), back(dv)], axis=-1)


@pytest.mark.parametrize("shape", [(2, 128, 2, 64), (1, 512, 3, 128), (3, 37, 2, 128), (2, 200, 1, 64),
                                   (1, 1, 2, 64), (1, 1000, 2, 128), (2, 2048, 2, 128),
                                   (1, 4100, 1, 128), (1, 2500, 2, 64), (5, 129, 3, 128), (1, 191, 1, 64),
                                   (2, 70, 3, 32)])       # a head size only the direct kernels take
def test_attention_bf16(shape):
    _attention_case(shape, 1.5)


@pytest.mark.parametrize("shape", [(1, 300, 2, 128), (2, 200, 2, 64), (1, 1100, 1, 128)])
def test_attention_bf16_peaked_scores(shape):
    """Scores with a standard deviation of several tens: nearly one-hot softmax rows, the running reference of the
    exponentials is raised again and again along a row, earlier keys underflow to exact zeros."""
    _attention_case(shape, 6.0)


def _attention_case(shape, std):
    B, S, H, dh = shape
    lib = _attn_lib()
    d = H * dh
    qkv = _bf(synth.normal(S + dh, "qkv", (B, S, 3 * d), std=std))
    dout = _bf(synth.normal(S + dh, "dout", (B, S, d)))
    ro, rlse, rdqkv = _attn_ref(qkv.double().numpy(), dout.double().numpy(), B, S, H, dh)
    qd, dod = qkv.cuda(), dout.cuda()
    o = torch.full((B, S, d), 9.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, H, S), 9.0, dtype=torch.float32, device="cuda")
    assert lib.swarm_kernel_attention_fwd(1, qd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, S, H, dh, None) == 0
    torch.cuda.synchronize()
    eo = np.max(np.abs(o.double().cpu().numpy() - ro)) / np.max(np.abs(ro))
    el = np.max(np.abs(lse.double().cpu().numpy() - rlse))
    assert eo < 1e-2, eo
    assert el < 2e-2, el
    delta = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    dqkv = torch.full((B, S, 3 * d), 9.0, dtype=torch.bfloat16, device="cuda")
    assert lib.swarm_kernel_attention_bwd(1, qd.data_ptr(), o.data_ptr(), dod.data_ptr(), lse.data_ptr(),
                                          delta.data_ptr(), dqkv.data_ptr(), B, S, H, dh, None) == 0
    torch.cuda.synchronize()
    got = dqkv.double().cpu().numpy()
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        den = max(np.max(np.abs(rdqkv[..., sl])), 1e-3 * np.max(np.abs(rdqkv)))   # S = 1 has dq = dk = 0 exactly
        e = np.max(np.abs(got[..., sl] - rdqkv[..., sl])) / den
        assert e < 1.5e-2, (name, e)
