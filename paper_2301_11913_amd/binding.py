"""ctypes binding of the C ABI in include/swarm_stage.h (argument marshalling only)."""
from __future__ import annotations

import contextlib
import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

SWARM_F32, SWARM_BF16 = 0, 1
SWARM_BLOCK_GELU, SWARM_BLOCK_ROTARY_GEGLU = 0, 1
PARAM_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")
EXPORTED_SYMBOLS = ("swarm_stage_workspace_bytes", "swarm_stage_forward", "swarm_stage_backward",
                    "swarm_codec_encode", "swarm_codec_decode", "swarm_status_string",
                    "swarm_stage_coded_workspace_bytes", "swarm_stage_forward_coded", "swarm_stage_backward_coded",
                    "swarm_boundary_workspace_bytes", "swarm_compress_forward", "swarm_compress_backward",
                    "swarm_decompress_forward", "swarm_decompress_backward",
                    "swarm_embedding_forward", "swarm_embedding_backward", "swarm_head_workspace_bytes",
                    "swarm_head_loss", "swarm_head_loss_backward",
                    "swarm_lamb_workspace_bytes", "swarm_lamb_step", "swarm_lamb_step_static",
                    "swarm_codec_encode_s16", "swarm_codec_decode_s16",
                    "swarm_stage_forward_coded_s16", "swarm_stage_backward_coded_s16")
SWARM_COMPRESS_BOTTLENECK, SWARM_COMPRESS_MAXOUT = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))


class SwarmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, swarm_status_string(status), status))


class _Config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32),
                ("n_layers", C.c_int32), ("n_repeat", C.c_int32), ("batch", C.c_int32),
                ("seq", C.c_int32), ("dtype", C.c_int32), ("ln_eps", C.c_float), ("block_kind", C.c_int32)]


class _BlockPtrs(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in PARAM_FIELDS]


class _BoundaryConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("d_comp", C.c_int32), ("kind", C.c_int32), ("tokens", C.c_int32),
                ("dtype", C.c_int32), ("ln_eps", C.c_float)]


class _Ptrs3(C.Structure):       # swarm_compress_params / _grads and swarm_decompress_params / _grads
    _fields_ = [("ln_g", C.c_void_p), ("ln_b", C.c_void_p), ("w", C.c_void_p)]


class BoundaryConfig:
    """Host-side description of a compressed stage boundary (mirrors swarm_boundary_config)."""

    def __init__(self, d_model, d_comp, kind, tokens, dtype, ln_eps=1e-5):
        if isinstance(kind, str):
            kind = {"bottleneck": SWARM_COMPRESS_BOTTLENECK, "maxout": SWARM_COMPRESS_MAXOUT}[kind]
        if isinstance(dtype, str):
            dtype = {"f32": SWARM_F32, "bf16": SWARM_BF16}[dtype]
        elif isinstance(dtype, torch.dtype):
            dtype = {torch.float32: SWARM_F32, torch.bfloat16: SWARM_BF16}[dtype]
        self.c = _BoundaryConfig(d_model, d_comp, kind, tokens, dtype, ln_eps)


class _HeadConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("vocab", C.c_int32), ("vocab_rows", C.c_int32), ("tokens", C.c_int32),
                ("dtype", C.c_int32), ("ln_eps", C.c_float)]


class HeadConfig:
    """Host-side description of the language-modelling head (mirrors swarm_head_config)."""

    def __init__(self, d_model, vocab, vocab_rows, tokens, dtype, ln_eps=1e-5):
        if isinstance(dtype, str):
            dtype = {"f32": SWARM_F32, "bf16": SWARM_BF16}[dtype]
        elif isinstance(dtype, torch.dtype):
            dtype = {torch.float32: SWARM_F32, torch.bfloat16: SWARM_BF16}[dtype]
        self.c = _HeadConfig(d_model, vocab, vocab_rows, tokens, dtype, ln_eps)


class _LambConfig(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("grad_scale", C.c_float), ("step", C.c_int32)]


class StageConfig:
    """Host-side description of a stage (mirrors swarm_stage_config)."""

    def __init__(self, d_model, n_heads, d_ffn, n_layers, n_repeat, batch, seq, dtype, ln_eps=1e-5,
                 block_kind=SWARM_BLOCK_GELU):
        if isinstance(block_kind, str):
            block_kind = {"gelu": SWARM_BLOCK_GELU, "rotary_geglu": SWARM_BLOCK_ROTARY_GEGLU}[block_kind]
        if isinstance(dtype, str):
            dtype = {"f32": SWARM_F32, "bf16": SWARM_BF16}[dtype]
        elif isinstance(dtype, torch.dtype):
            dtype = {torch.float32: SWARM_F32, torch.bfloat16: SWARM_BF16}[dtype]
        self.c = _Config(d_model, n_heads, d_ffn, n_layers, n_repeat, batch, seq, dtype, ln_eps, block_kind)

    @property
    def torch_dtype(self):
        return torch.float32 if self.c.dtype == SWARM_F32 else torch.bfloat16


def lib_path() -> str:
    return os.environ.get("SWARM_STAGE_LIB", os.path.join(_PKG, "libswarm_stage.so"))


def hooks_lib_path() -> str:
    return os.environ.get("SWARM_HOOKS_LIB", os.path.join(_PKG, "libswarm_hooks.so"))


_lib = None
_hooks_lib = None


def load_library():
    """Load libswarm_stage.so; raises if it has not been built (there is no fallback).  Inside a
    `with using_hooks_library():` block the instrumented build is returned instead."""
    global _lib
    if _lib is not None:
        return _lib
    _lib = _open(lib_path())
    return _lib


def load_hooks_library():
    """Load libswarm_hooks.so: the same sources plus the single-kernel entry points (swarm_kernel_*), the per-launch
    GEMM timer and the micro-benchmarks.  For tests and measurements only; the product is libswarm_stage.so."""
    global _hooks_lib
    if _hooks_lib is None:
        _hooks_lib = _open(hooks_lib_path())
    return _hooks_lib


@contextlib.contextmanager
def using_hooks_library():
    """Route every binding call inside the block to libswarm_hooks.so (bench.py times GEMM launches this way)."""
    global _lib
    product = load_library()
    _lib = load_hooks_library()
    try:
        yield _lib
    finally:
        _lib = product


def _open(path):
    if not os.path.exists(path):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2301_11913_amd.build` "
            "(the library has no CPU fallback)" % path)
    lib = C.CDLL(path)
    lib.swarm_stage_workspace_bytes.restype = C.c_size_t
    lib.swarm_stage_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int]
    lib.swarm_stage_forward.restype = C.c_int
    lib.swarm_stage_forward.argtypes = [C.POINTER(_Config), C.POINTER(_BlockPtrs), C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    lib.swarm_stage_backward.restype = C.c_int
    lib.swarm_stage_backward.argtypes = [C.POINTER(_Config), C.POINTER(_BlockPtrs), C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.POINTER(_BlockPtrs), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.swarm_codec_encode.restype = C.c_int
    lib.swarm_codec_encode.argtypes = [C.c_void_p, C.c_int32, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p]
    lib.swarm_codec_decode.restype = C.c_int
    lib.swarm_codec_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_int32,
                                       C.c_void_p]
    lib.swarm_codec_encode_s16.restype = C.c_int
    lib.swarm_codec_encode_s16.argtypes = lib.swarm_codec_encode.argtypes
    lib.swarm_codec_decode_s16.restype = C.c_int
    lib.swarm_codec_decode_s16.argtypes = lib.swarm_codec_decode.argtypes
    lib.swarm_stage_coded_workspace_bytes.restype = C.c_size_t
    lib.swarm_stage_coded_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int]
    lib.swarm_stage_forward_coded.restype = C.c_int
    lib.swarm_stage_forward_coded.argtypes = [C.POINTER(_Config), C.POINTER(_BlockPtrs)] + [C.c_void_p] * 6 + \
                                             [C.c_size_t, C.c_void_p]
    lib.swarm_stage_backward_coded.restype = C.c_int
    lib.swarm_stage_backward_coded.argtypes = [C.POINTER(_Config), C.POINTER(_BlockPtrs)] + [C.c_void_p] * 5 + \
                                              [C.POINTER(_BlockPtrs), C.c_void_p, C.c_size_t, C.c_void_p]
    for suffix in ("", "_s16"):
        getattr(lib, "swarm_stage_forward_coded" + suffix).restype = C.c_int
        getattr(lib, "swarm_stage_forward_coded" + suffix).argtypes = lib.swarm_stage_forward_coded.argtypes
        getattr(lib, "swarm_stage_backward_coded" + suffix).restype = C.c_int
        getattr(lib, "swarm_stage_backward_coded" + suffix).argtypes = lib.swarm_stage_backward_coded.argtypes
    lib.swarm_boundary_workspace_bytes.restype = C.c_size_t
    lib.swarm_boundary_workspace_bytes.argtypes = [C.POINTER(_BoundaryConfig), C.c_int, C.c_int]
    for name in ("swarm_compress_forward", "swarm_decompress_forward"):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [C.POINTER(_BoundaryConfig), C.POINTER(_Ptrs3), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                       C.c_void_p]
    for name in ("swarm_compress_backward", "swarm_decompress_backward"):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [C.POINTER(_BoundaryConfig), C.POINTER(_Ptrs3), C.c_void_p, C.c_void_p, C.c_void_p,
                       C.POINTER(_Ptrs3), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.swarm_embedding_forward.restype = C.c_int
    lib.swarm_embedding_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p]
    lib.swarm_embedding_backward.restype = C.c_int
    lib.swarm_embedding_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p]
    lib.swarm_head_workspace_bytes.restype = C.c_size_t
    lib.swarm_head_workspace_bytes.argtypes = [C.POINTER(_HeadConfig), C.c_int]
    lib.swarm_head_loss.restype = C.c_int
    lib.swarm_head_loss.argtypes = [C.POINTER(_HeadConfig), C.POINTER(_Ptrs3), C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.swarm_head_loss_backward.restype = C.c_int
    lib.swarm_head_loss_backward.argtypes = [C.POINTER(_HeadConfig), C.POINTER(_Ptrs3), C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_Ptrs3), C.c_void_p,
                                             C.c_size_t, C.c_void_p]
    lib.swarm_lamb_workspace_bytes.restype = C.c_size_t
    lib.swarm_lamb_workspace_bytes.argtypes = [C.c_size_t]
    lib.swarm_lamb_step.restype = C.c_int
    lib.swarm_lamb_step.argtypes = [C.POINTER(_LambConfig), C.c_size_t, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.swarm_lamb_step_static.restype = C.c_int
    lib.swarm_lamb_step_static.argtypes = [C.POINTER(_LambConfig), C.c_size_t, C.c_void_p, C.c_void_p, C.c_int32,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.swarm_status_string.restype = C.c_char_p
    lib.swarm_status_string.argtypes = [C.c_int]
    return lib


def swarm_status_string(status: int) -> str:
    return load_library().swarm_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to the stage library must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SWARM_F32
    if t.dtype == torch.bfloat16:
        return SWARM_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _block_array(blocks: Sequence[Dict[str, torch.Tensor]]):
    arr = (_BlockPtrs * len(blocks))()
    for i, b in enumerate(blocks):
        for k in PARAM_FIELDS:
            setattr(arr[i], k, _ptr(b[k]))
    return arr


def swarm_stage_workspace_bytes(cfg: StageConfig, for_backward: bool) -> int:
    return int(load_library().swarm_stage_workspace_bytes(C.byref(cfg.c), 1 if for_backward else 0))


def swarm_stage_forward(cfg: StageConfig, params: List[Dict[str, torch.Tensor]], x_in: torch.Tensor,
                        x_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    st = load_library().swarm_stage_forward(C.byref(cfg.c), _block_array(params), _ptr(x_in), _ptr(x_out),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_stage_forward")


def swarm_stage_backward(cfg: StageConfig, params: List[Dict[str, torch.Tensor]], x_in: torch.Tensor,
                         grad_out: torch.Tensor, grad_in: torch.Tensor,
                         grad_params: List[Dict[str, torch.Tensor]], workspace: torch.Tensor,
                         stream=None) -> None:
    for g in grad_params:
        for k in PARAM_FIELDS:
            if g[k].dtype != torch.float32:
                raise TypeError("grad_params must be fp32")
    st = load_library().swarm_stage_backward(C.byref(cfg.c), _block_array(params), _ptr(x_in), _ptr(grad_out),
                                             _ptr(grad_in), _block_array(grad_params), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_stage_backward")


def swarm_codec_encode(tensor: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, block: int = 64,
                       stream=None) -> None:
    if codes.dtype != torch.int8 or scales.dtype != torch.float32:
        raise TypeError("codes must be int8 and scales fp32")
    st = load_library().swarm_codec_encode(_ptr(tensor), _dtype_code(tensor), tensor.numel(), block, _ptr(codes),
                                           _ptr(scales), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_codec_encode")


def swarm_codec_decode(codes: torch.Tensor, scales: torch.Tensor, tensor: torch.Tensor, block: int = 64,
                       stream=None) -> None:
    if codes.dtype != torch.int8 or scales.dtype != torch.float32:
        raise TypeError("codes must be int8 and scales fp32")
    st = load_library().swarm_codec_decode(_ptr(codes), _ptr(scales), tensor.numel(), block, _ptr(tensor),
                                           _dtype_code(tensor), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_codec_decode")


def swarm_codec_encode_s16(tensor: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, block: int = 64,
                           stream=None) -> None:
    """scales: int16 / uint16 tensor receiving bf16 bit patterns (or a bf16 tensor, which is the same memory)."""
    if codes.dtype != torch.int8 or scales.element_size() != 2:
        raise TypeError("codes must be int8 and scales a 16-bit tensor")
    st = load_library().swarm_codec_encode_s16(_ptr(tensor), _dtype_code(tensor), tensor.numel(), block, _ptr(codes),
                                               _ptr(scales), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_codec_encode_s16")


def swarm_codec_decode_s16(codes: torch.Tensor, scales: torch.Tensor, tensor: torch.Tensor, block: int = 64,
                           stream=None) -> None:
    if codes.dtype != torch.int8 or scales.element_size() != 2:
        raise TypeError("codes must be int8 and scales a 16-bit tensor")
    st = load_library().swarm_codec_decode_s16(_ptr(codes), _ptr(scales), tensor.numel(), block, _ptr(tensor),
                                               _dtype_code(tensor), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_codec_decode_s16")


def swarm_stage_coded_workspace_bytes(cfg: StageConfig, for_backward: bool) -> int:
    return int(load_library().swarm_stage_coded_workspace_bytes(C.byref(cfg.c), 1 if for_backward else 0))


def _scale_suffix(*scales: torch.Tensor) -> str:
    """"" for fp32 block scales, "_s16" for 16-bit ones (all scale tensors of a call must agree)."""
    sizes = {t.element_size() for t in scales}
    if sizes == {4} and all(t.dtype == torch.float32 for t in scales):
        return ""
    if sizes == {2}:
        return "_s16"
    raise TypeError("block scales must be all fp32 or all 16-bit tensors")


def swarm_stage_forward_coded(cfg: StageConfig, params: List[Dict[str, torch.Tensor]], x_codes: torch.Tensor,
                              x_scales: torch.Tensor, x_dec: torch.Tensor, y_codes: torch.Tensor,
                              y_scales: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """fp32 scale tensors call swarm_stage_forward_coded, 16-bit ones swarm_stage_forward_coded_s16."""
    name = "swarm_stage_forward_coded" + _scale_suffix(x_scales, y_scales)
    st = getattr(load_library(), name)(C.byref(cfg.c), _block_array(params), _ptr(x_codes), _ptr(x_scales),
                                       _ptr(x_dec), _ptr(y_codes), _ptr(y_scales), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, name)


def swarm_stage_backward_coded(cfg: StageConfig, params: List[Dict[str, torch.Tensor]], x_in: torch.Tensor,
                               g_codes: torch.Tensor, g_scales: torch.Tensor, gin_codes: torch.Tensor,
                               gin_scales: torch.Tensor, grad_params: List[Dict[str, torch.Tensor]],
                               workspace: torch.Tensor, stream=None) -> None:
    name = "swarm_stage_backward_coded" + _scale_suffix(g_scales, gin_scales)
    st = getattr(load_library(), name)(C.byref(cfg.c), _block_array(params), _ptr(x_in), _ptr(g_codes),
                                       _ptr(g_scales), _ptr(gin_codes), _ptr(gin_scales),
                                       _block_array(grad_params), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, name)


def _ptrs3(d: Dict[str, torch.Tensor], wkey: str):
    return _Ptrs3(_ptr(d["ln_g"]), _ptr(d["ln_b"]), _ptr(d.get(wkey)))


def _check_f32(grads: Dict[str, torch.Tensor]):
    for g in grads.values():
        if g is not None and g.dtype != torch.float32:
            raise TypeError("parameter gradients must be fp32")


def swarm_boundary_workspace_bytes(cfg: BoundaryConfig, decompress: bool, for_backward: bool) -> int:
    return int(load_library().swarm_boundary_workspace_bytes(C.byref(cfg.c), int(decompress), int(for_backward)))


def swarm_compress_forward(cfg: BoundaryConfig, params: Dict[str, torch.Tensor], y: torch.Tensor, z: torch.Tensor,
                           workspace: torch.Tensor, stream=None) -> None:
    st = load_library().swarm_compress_forward(C.byref(cfg.c), C.byref(_ptrs3(params, "w_c")), _ptr(y), _ptr(z),
                                               _ptr(workspace), workspace.numel() * workspace.element_size(),
                                               _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_compress_forward")


def swarm_compress_backward(cfg: BoundaryConfig, params: Dict[str, torch.Tensor], y: torch.Tensor, dz: torch.Tensor,
                            dy: torch.Tensor, grads: Dict[str, torch.Tensor], workspace: torch.Tensor,
                            stream=None) -> None:
    _check_f32(grads)
    st = load_library().swarm_compress_backward(C.byref(cfg.c), C.byref(_ptrs3(params, "w_c")), _ptr(y), _ptr(dz),
                                                _ptr(dy), C.byref(_ptrs3(grads, "w_c")), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_compress_backward")


def swarm_decompress_forward(cfg: BoundaryConfig, params: Dict[str, torch.Tensor], z: torch.Tensor, x: torch.Tensor,
                             workspace: torch.Tensor, stream=None) -> None:
    st = load_library().swarm_decompress_forward(C.byref(cfg.c), C.byref(_ptrs3(params, "w_d")), _ptr(z), _ptr(x),
                                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                 _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_decompress_forward")


def swarm_decompress_backward(cfg: BoundaryConfig, params: Dict[str, torch.Tensor], z: torch.Tensor, dx: torch.Tensor,
                              dz: torch.Tensor, grads: Dict[str, torch.Tensor], workspace: torch.Tensor,
                              stream=None) -> None:
    _check_f32(grads)
    st = load_library().swarm_decompress_backward(C.byref(cfg.c), C.byref(_ptrs3(params, "w_d")), _ptr(z), _ptr(dx),
                                                  _ptr(dz), C.byref(_ptrs3(grads, "w_d")), _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_decompress_backward")


def swarm_embedding_forward(tokens: torch.Tensor, table: torch.Tensor, vocab: int, x: torch.Tensor,
                            stream=None) -> None:
    if tokens.dtype != torch.int32:
        raise TypeError("token ids must be int32")
    st = load_library().swarm_embedding_forward(_ptr(tokens), _ptr(table), _dtype_code(table), tokens.numel(), vocab,
                                                table.shape[1], _ptr(x), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_embedding_forward")


def swarm_embedding_backward(tokens: torch.Tensor, dx: torch.Tensor, vocab: int, grad_table: torch.Tensor,
                             stream=None) -> None:
    if tokens.dtype != torch.int32 or grad_table.dtype != torch.float32:
        raise TypeError("token ids must be int32 and grad_table fp32")
    st = load_library().swarm_embedding_backward(_ptr(tokens), _ptr(dx), _dtype_code(dx), tokens.numel(), vocab,
                                                 dx.shape[1], _ptr(grad_table), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_embedding_backward")


def swarm_head_workspace_bytes(cfg: HeadConfig, for_backward: bool) -> int:
    return int(load_library().swarm_head_workspace_bytes(C.byref(cfg.c), int(for_backward)))


def swarm_head_loss(cfg: HeadConfig, params: Dict[str, torch.Tensor], x: torch.Tensor, targets: torch.Tensor,
                    loss: torch.Tensor, token_loss: Optional[torch.Tensor], workspace: torch.Tensor,
                    stream=None) -> None:
    if targets.dtype != torch.int32 or loss.dtype != torch.float32:
        raise TypeError("targets must be int32 and loss fp32")
    st = load_library().swarm_head_loss(C.byref(cfg.c), C.byref(_ptrs3(params, "w_vocab")), _ptr(x), _ptr(targets),
                                        _ptr(loss), _ptr(token_loss), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_head_loss")


def swarm_head_loss_backward(cfg: HeadConfig, params: Dict[str, torch.Tensor], x: torch.Tensor, targets: torch.Tensor,
                             loss: torch.Tensor, token_loss: Optional[torch.Tensor], dx: torch.Tensor,
                             grads: Dict[str, torch.Tensor], workspace: torch.Tensor, stream=None) -> None:
    if targets.dtype != torch.int32 or loss.dtype != torch.float32:
        raise TypeError("targets must be int32 and loss fp32")
    _check_f32(grads)
    st = load_library().swarm_head_loss_backward(C.byref(cfg.c), C.byref(_ptrs3(params, "w_vocab")), _ptr(x),
                                                 _ptr(targets), _ptr(loss), _ptr(token_loss), _ptr(dx),
                                                 C.byref(_ptrs3(grads, "w_vocab")), _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_head_loss_backward")


def swarm_lamb_workspace_bytes(n_elems: int) -> int:
    return int(load_library().swarm_lamb_workspace_bytes(n_elems))


def swarm_lamb_step(master: torch.Tensor, param: Optional[torch.Tensor], grad: torch.Tensor, m: torch.Tensor,
                    v: torch.Tensor, step: int, workspace: torch.Tensor, lr: float = 1e-3, beta1: float = 0.9,
                    beta2: float = 0.95, eps: float = 1e-6, weight_decay: float = 0.01, grad_scale: float = 1.0,
                    trust_ratio: Optional[torch.Tensor] = None, stream=None) -> None:
    for t in (master, grad, m, v):
        if t.dtype != torch.float32:
            raise TypeError("master weights, gradient and moments must be fp32")
    cfg = _LambConfig(lr, beta1, beta2, eps, weight_decay, grad_scale, step)
    st = load_library().swarm_lamb_step(C.byref(cfg), master.numel(), _ptr(master), _ptr(param),
                                        _dtype_code(param) if param is not None else SWARM_F32, _ptr(grad), _ptr(m),
                                        _ptr(v), _ptr(trust_ratio), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_lamb_step")


SWARM_LAMB_STATIC_MAX_ELEMS = 1 << 24


def swarm_lamb_step_static(master: torch.Tensor, param: Optional[torch.Tensor], grad: torch.Tensor, m: torch.Tensor,
                           v: torch.Tensor, step: int, lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.95,
                           eps: float = 1e-6, weight_decay: float = 0.01, grad_scale: float = 1.0,
                           trust_ratio: Optional[torch.Tensor] = None, stream=None) -> None:
    for t in (master, grad, m, v):
        if t.dtype != torch.float32:
            raise TypeError("master weights, gradient and moments must be fp32")
    cfg = _LambConfig(lr, beta1, beta2, eps, weight_decay, grad_scale, step)
    st = load_library().swarm_lamb_step_static(C.byref(cfg), master.numel(), _ptr(master), _ptr(param),
                                               _dtype_code(param) if param is not None else SWARM_F32, _ptr(grad),
                                               _ptr(m), _ptr(v), _ptr(trust_ratio), _stream(stream))
    if st != 0:
        raise SwarmError(st, "swarm_lamb_step_static")
