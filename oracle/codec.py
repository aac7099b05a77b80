"""Oracle for the 8-bit blockwise boundary codec (TEST INFRASTRUCTURE, not product code).

The paper (appendix "Compression-Aware Architectures", paragraph "Quantized
activations") sends activations and activation gradients between pipeline stages
with dynamic 8-bit quantisation and blockwise scaling, cutting traffic roughly
2x against 16-bit and 4x against 32-bit tensors.  It does not spell the scheme
out; the reading implemented here (and by the HIP kernels) is uniform symmetric
int8 with one run-time scale per block of 64 consecutive elements of the
flattened tensor:

  encode, per block, all in IEEE fp32 (one rounding per operation):
    A      = max_i |x_i|
    scale  = A / 127
    code_i = 0                                        if scale == 0
           = clamp(round_half_even(x_i / scale), -127, 127)   otherwise
  decode:
    y_i    = float(code_i) * scale, then rounded to the tensor's dtype.

Stored per block: 64 int8 codes + one fp32 scale (1.0625 B/element).
Plain numpy, one array operation per step above; no blocking or fusion.

Option scale_bits=16 (the paragraph's "about 2x against 16-bit" needs less than the 6 % that fp32 scales add):
the scale is rounded once more, to bf16 (nearest even; bf16 because it keeps fp32's exponent range, so the tiny
scales of gradient tensors survive), BEFORE the codes are computed, and is stored as its 16 bit pattern
(1.03125 B/element).  Codes divide by that rounded scale: one bf16 rounding moves it by at most 2^-8 relative, so
|x/scale| stays below 127.5, the largest element still gets +-127 and its round-trip error stays under half a
step like everyone else's; a scale that rounds to zero (below 2^-134) encodes its block as zeros.

Pins (tests/test_oracle_codec.py): exact-rational re-computation of every step
(both scale widths), the half-step round-trip bound, absmax -> +-127, zero blocks,
idempotence, all finite bf16 bit patterns, the traffic ratios quoted by the paper.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 values (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def _scale(a, scale_bits):
    """absmax (fp32 scalar or array) -> the scale the codes divide by, as fp32."""
    s = a / np.float32(127.0)                                # one fp32 division
    if scale_bits == 16:
        s = bf16_bits_to_f32(f32_to_bf16_bits(s))            # second rounding, to bf16
    elif scale_bits != 32:
        raise ValueError(scale_bits)
    return s


def encode(x: np.ndarray, block: int = 64, scale_bits: int = 32):
    """x: flat fp32 array (bf16 inputs are passed already widened, which is exact).

    Returns (codes int8 [n], scales [ceil(n/block)]: fp32, or uint16 bf16 bit patterns with scale_bits=16)."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    n = x.size
    nb = (n + block - 1) // block
    codes = np.zeros(n, dtype=np.int8)
    scales = np.zeros(nb, dtype=np.float32)
    full = n // block
    if full:
        xb = x[: full * block].reshape(full, block)
        a = np.max(np.abs(xb), axis=1)                       # A
        s = _scale(a, scale_bits)
        scales[:full] = s
        safe = np.where(s == 0, np.float32(1.0), s)
        q = np.rint(xb / safe[:, None])                      # fp32 division, ties to even
        q = np.clip(q, np.float32(-127.0), np.float32(127.0))
        q = np.where((s == 0)[:, None], np.float32(0.0), q)
        codes[: full * block] = q.astype(np.int8).reshape(-1)
    if n > full * block:                                     # ragged last block
        xt = x[full * block:]
        s = _scale(np.float32(np.max(np.abs(xt))).reshape(1), scale_bits)[0]
        scales[full] = s
        if s != 0:
            q = np.clip(np.rint(xt / s), np.float32(-127.0), np.float32(127.0))
            codes[full * block:] = q.astype(np.int8)
    return codes, (f32_to_bf16_bits(scales) if scale_bits == 16 else scales)     # exact: already bf16 values


def decode(codes: np.ndarray, scales: np.ndarray, block: int = 64, out: str = "f32") -> np.ndarray:
    """scales: fp32, or uint16 bf16 bit patterns (16-bit option).
    Returns fp32 values (out="f32") or bf16 bit patterns as uint16 (out="bf16")."""
    codes = np.ascontiguousarray(codes, dtype=np.int8).reshape(-1)
    n = codes.size
    scales = np.ascontiguousarray(scales)
    if scales.dtype == np.uint16:
        scales = bf16_bits_to_f32(scales)
    s = np.repeat(np.ascontiguousarray(scales, dtype=np.float32), block)[:n]
    y = codes.astype(np.float32) * s                         # one fp32 multiplication
    if out == "f32":
        return y
    if out == "bf16":
        return f32_to_bf16_bits(y)
    raise ValueError(out)
