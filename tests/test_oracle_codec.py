"""Pins for the codec oracle: every step re-derived in exact rational arithmetic,
the half-step bound, and the degenerate cases.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import codec
import swarm_synth as synth

HERE = os.path.dirname(__file__)


def _round_to_f32(fr: Fraction) -> np.float32:
    """Correctly rounded (nearest-even) fp32 of an exact rational, via exact integer arithmetic."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    # find e with 2^e <= fr < 2^(e+1)
    e = fr.numerator.bit_length() - fr.denominator.bit_length()
    if Fraction(2) ** e > fr:
        e -= 1
    if Fraction(2) ** (e + 1) <= fr:
        e += 1
    e_q = max(e, -126) - 23                     # exponent of one ulp (subnormals share 2^-149)
    q = fr / (Fraction(2) ** e_q)
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    val = Fraction(n) * (Fraction(2) ** e_q)
    return np.float32(sign * float(val))         # val is exactly representable


def _exact_encode_block(xs):
    """Independent re-statement with exact rationals + explicit fp32 roundings."""
    fx = [Fraction(float(v)) for v in xs]
    A = max(abs(v) for v in fx)
    scale = _round_to_f32(A / 127)
    if scale == 0:
        return [0] * len(xs), scale
    fs = Fraction(float(scale))
    out = []
    for v in fx:
        qf = Fraction(float(_round_to_f32(v / fs)))      # fp32 quotient
        n = qf.numerator // qf.denominator               # floor
        rem = qf - n
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
            n += 1
        out.append(int(max(-127, min(127, n))))
    return out, scale


def test_round_helper_matches_numpy_division():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(200).astype(np.float32)
    b = (rng.standard_normal(200).astype(np.float32) + np.float32(3.0))
    for x, y in zip(a, b):
        assert _round_to_f32(Fraction(float(x)) / Fraction(float(y))) == np.float32(x) / np.float32(y)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("std", [1.0, 1e-2, 3e-5])
def test_encode_matches_exact_rational(bf16, std):
    x = synth.codec_tensor(7, 64 * 24 + 17, std=std, bf16=bf16)
    codes, scales = codec.encode(x, 64)
    nb = (x.size + 63) // 64
    assert scales.shape == (nb,) and codes.shape == (x.size,)
    for b in range(nb):
        blk = x[b * 64:(b + 1) * 64]
        ec, es = _exact_encode_block(blk)
        assert es == scales[b]
        assert ec == codes[b * 64:(b + 1) * 64].tolist()


def test_ties_round_to_even():
    # absmax 127 -> scale exactly 1, so x/scale = x: halves must go to the even neighbour
    x = np.zeros(64, dtype=np.float32)
    x[0] = 127.0
    x[1:9] = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5]
    codes, scales = codec.encode(x)
    assert scales[0] == np.float32(1.0)
    assert codes[:9].tolist() == [127, 0, 2, 2, 0, -2, -2, 4, 126]


def test_half_step_bound_and_extremes():
    for std, bf in [(1.0, False), (1.0, True), (1e-2, True), (40.0, False)]:
        x = synth.codec_tensor(11, 64 * 512, std=std, bf16=bf)
        codes, scales = codec.encode(x)
        y = codec.decode(codes, scales)
        s = np.repeat(scales.astype(np.float64), 64)
        err = np.abs(x.astype(np.float64) - y.astype(np.float64))
        # half a quantisation step, plus the rounding of the fp32 division and multiplication
        assert np.all(err <= s * (0.5 + 127 * 2.0 ** -22))
        xb = x.reshape(-1, 64)
        cb = codes.reshape(-1, 64)
        am = np.argmax(np.abs(xb), axis=1)
        rows = np.arange(xb.shape[0])
        assert np.all(np.abs(cb[rows, am].astype(np.int32)) == 127)
        assert np.all(np.sign(cb[rows, am]) == np.sign(xb[rows, am]))
        assert cb.min() >= -127


def test_zero_block_and_ragged_tail_and_empty():
    x = synth.codec_tensor(3, 64 * 3 + 5)
    x[64:128] = 0.0
    codes, scales = codec.encode(x)
    assert scales[1] == 0 and not codes[64:128].any()
    assert np.all(codec.decode(codes, scales)[64:128] == 0)
    # the 5-element tail is a block of its own
    ec, es = _exact_encode_block(x[192:])
    assert es == scales[3] and ec == codes[192:].tolist()
    c0, s0 = codec.encode(np.zeros(0, dtype=np.float32))
    assert c0.size == 0 and s0.size == 0
    assert codec.decode(c0, s0).size == 0


def test_reencode_is_idempotent():
    x = synth.codec_tensor(5, 64 * 256)
    c1, s1 = codec.encode(x)
    c2, s2 = codec.encode(codec.decode(c1, s1))
    assert np.array_equal(c1, c2)
    # scale can move by rounding of 127*s/127 only
    assert np.allclose(s1, s2, rtol=2.0 ** -22, atol=0)


def test_all_finite_bf16_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = codec.bf16_bits_to_f32(bits)
    fin = np.isfinite(vals)
    bits, vals = bits[fin], vals[fin]
    # bf16 round trip is the identity on bf16 values
    assert np.array_equal(codec.f32_to_bf16_bits(vals), bits)
    # (a) every value as a single-element block: code = +-127 (or 0 when the scale underflows)
    codes, scales = codec.encode(vals, block=1)
    nz = scales != 0
    assert np.all(np.abs(codes[nz].astype(np.int32)) == 127)
    assert np.all(codes[~nz] == 0)
    dec = codec.decode(codes, scales, block=1)
    # two fp32 roundings; a subnormal scale is only exact to half of 2^-149, times 127
    assert np.all(np.abs(dec[nz].astype(np.float64) - vals[nz])
                  <= np.abs(vals[nz].astype(np.float64)) * 2.0 ** -22 + 127 * 2.0 ** -150)
    # (b) values inside blocks of fixed absmax 2.0: compare with exact rationals on a sample
    inside = vals[np.abs(vals) <= 2.0]
    pad = (-inside.size) % 63
    inside = np.concatenate([inside, np.zeros(pad, dtype=np.float32)]).reshape(-1, 63)
    blocks = np.concatenate([np.full((inside.shape[0], 1), 2.0, dtype=np.float32), inside], axis=1)
    codes, scales = codec.encode(blocks.reshape(-1))
    assert np.all(scales == np.float32(2.0) / np.float32(127.0))
    cb = codes.reshape(-1, 64)
    for r in range(0, blocks.shape[0], 7):
        ec, _ = _exact_encode_block(blocks[r])
        assert ec == cb[r].tolist()
    # monotone: larger value never gets a smaller code
    order = np.argsort(blocks.reshape(-1), kind="stable")
    assert np.all(np.diff(codes.astype(np.int32)[order]) >= 0)


def test_bf16_output_rounding():
    x = synth.codec_tensor(9, 64 * 64, bf16=True)
    codes, scales = codec.encode(x)
    y32 = codec.decode(codes, scales, out="f32")
    yb = codec.decode(codes, scales, out="bf16")
    back = codec.bf16_bits_to_f32(yb).astype(np.float64)
    # nearest bf16: error at most half a bf16 ulp (2^-8 relative)
    assert np.all(np.abs(back - y32) <= np.abs(y32.astype(np.float64)) * 2.0 ** -8)
    import torch
    ref = torch.from_numpy(y32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ref, yb)


def test_traffic_ratio_matches_paper():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "codec_traffic.txt")) if not l.startswith("#")]
    per_elem = 1 + 4 / 64
    for src, approx in rows:
        ratio = float(src) / per_elem
        assert abs(ratio - float(approx)) / float(approx) < 0.07


# ------------------------------------------------------------------ 16-bit scales
def _round_to_bits(fr: Fraction, p: int, emin: int) -> Fraction:
    """Nearest-even rounding of an exact rational to a binary format with p significand bits (hidden bit
    included) and smallest normal exponent emin; exact integer arithmetic, subnormals included."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = fr.numerator.bit_length() - fr.denominator.bit_length()
    if Fraction(2) ** e > fr:
        e -= 1
    if Fraction(2) ** (e + 1) <= fr:
        e += 1
    ulp = Fraction(2) ** (max(e, emin) - (p - 1))
    q = fr / ulp
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return sign * n * ulp


def _exact_encode_block_s16(xs):
    fx = [Fraction(float(v)) for v in xs]
    A = max(abs(v) for v in fx)
    s32 = _round_to_bits(A / 127, 24, -126)                  # the fp32 division
    fs = _round_to_bits(s32, 8, -126)                        # then once more, to bf16
    if fs == 0:
        return [0] * len(xs), fs
    out = []
    for v in fx:
        qf = _round_to_bits(v / fs, 24, -126)
        n = qf.numerator // qf.denominator
        rem = qf - n
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
            n += 1
        out.append(int(max(-127, min(127, n))))
    return out, fs


def test_round_to_bits_helper_against_numpy_and_torch():
    import torch
    rng = np.random.default_rng(1)
    v = np.concatenate([rng.standard_normal(300) * 10.0 ** rng.integers(-42, 30, 300), [2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -135]])
    v32 = v.astype(np.float32)
    for x64, x32 in zip(v, v32):
        assert float(_round_to_bits(Fraction(float(x64)), 24, -126)) == float(x32)
    tb = torch.from_numpy(v32).to(torch.bfloat16).float().numpy()
    for x32, xb in zip(v32, tb):
        assert float(_round_to_bits(Fraction(float(x32)), 8, -126)) == float(xb)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("std", [1.0, 1e-2, 3e-5, 1e-38])
def test_encode_s16_matches_exact_rational(bf16, std):
    x = synth.codec_tensor(17, 64 * 24 + 17, std=std, bf16=bf16)
    codes, sbits = codec.encode(x, 64, scale_bits=16)
    assert sbits.dtype == np.uint16 and sbits.shape == ((x.size + 63) // 64,)
    sval = codec.bf16_bits_to_f32(sbits)
    for b in range(sbits.size):
        ec, es = _exact_encode_block_s16(x[b * 64:(b + 1) * 64])
        assert float(es) == float(sval[b])
        assert ec == codes[b * 64:(b + 1) * 64].tolist()


def test_s16_half_step_bound_extremes_and_fp32_path_untouched():
    for std, bf in [(1.0, False), (1.0, True), (1e-2, True), (40.0, False)]:
        x = synth.codec_tensor(12, 64 * 512, std=std, bf16=bf)
        codes, sbits = codec.encode(x, scale_bits=16)
        c32, s32 = codec.encode(x)
        sval = codec.bf16_bits_to_f32(sbits)
        assert np.all(np.abs(sval.astype(np.float64) - s32) <= s32.astype(np.float64) * 2.0 ** -8)   # one bf16 rounding
        assert s32.dtype == np.float32 and np.any(sval != s32)
        y = codec.decode(codes, sbits)
        s = np.repeat(sval.astype(np.float64), 64)
        err = np.abs(x.astype(np.float64) - y.astype(np.float64))
        assert np.all(err <= s * (0.5 + 127 * 2.0 ** -22))          # also for the largest element (127 * 2^-8 < 1/2)
        xb, cb = x.reshape(-1, 64), codes.reshape(-1, 64)
        am, rows = np.argmax(np.abs(xb), axis=1), np.arange(xb.shape[0])
        assert np.all(np.abs(cb[rows, am].astype(np.int32)) == 127) and cb.min() >= -127
        assert np.mean(codes != c32) < 0.2                          # same grid up to the scale's last bit


def test_s16_scale_flushes_to_zero_and_ragged_and_empty():
    x = np.zeros(64 * 2 + 3, dtype=np.float32)
    x[:64] = np.float32(2.0 ** -130)            # A / 127 = 2^-137 rounds to bf16 zero (half of the smallest
    x[64:128] = np.float32(1.5)                 # subnormal 2^-133 is 2^-134)
    x[128:] = [0.25, -1.0, 0.5]
    codes, sbits = codec.encode(x, scale_bits=16)
    assert sbits[0] == 0 and not codes[:64].any()
    assert codes[64] == 127 and codes[129] == -127
    ec, es = _exact_encode_block_s16(x[128:])
    assert ec == codes[128:].tolist()
    assert np.all(codec.decode(codes, sbits)[:64] == 0)
    c0, s0 = codec.encode(np.zeros(0, dtype=np.float32), scale_bits=16)
    assert c0.size == 0 and s0.size == 0 and s0.dtype == np.uint16


def test_s16_traffic_ratio_matches_paper():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "codec_traffic.txt")) if not l.startswith("#")]
    per_elem = 1 + 2 / 64
    for src, approx in rows:
        ratio = float(src) / per_elem
        assert abs(ratio - float(approx)) / float(approx) < 0.035   # twice as close to the quoted factors as fp32 scales
