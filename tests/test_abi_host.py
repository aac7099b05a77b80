"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2301_11913_amd as sw
from paper_2301_11913_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swarm_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sw.lib_path()):
        pytest.skip("libswarm_stage.so not built")
    return sw.load_library()


def test_exports_every_declared_symbol(lib):
    syms = _header_symbols()
    assert set(syms) == set(sw.EXPORTED_SYMBOLS)
    for s in syms:
        assert getattr(lib, s) is not None


def test_product_library_has_no_test_hooks(lib):
    """Single-kernel entry points, the GEMM launch timer and the micro-benchmarks live in libswarm_hooks.so only."""
    hooks = ("swarm_kernel_gemm", "swarm_kernel_gemm_ws", "swarm_kernel_gemm_stamped", "swarm_kernel_attention_fwd",
             "swarm_kernel_attention_bwd", "swarm_kernel_quantise_pairs", "swarm_kernel_timing_enable",
             "swarm_kernel_timing_collect", "swarm_microbench_mfma_rate", "swarm_microbench_lds_read")
    for s in hooks:
        assert not hasattr(lib, s), s
    if not os.path.exists(sw.hooks_lib_path()):
        pytest.skip("libswarm_hooks.so not built")
    hl = sw.load_hooks_library()
    for s in hooks + tuple(sw.EXPORTED_SYMBOLS):
        assert getattr(hl, s) is not None


def test_status_strings(lib):
    assert sw.swarm_status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert sw.swarm_status_string(code) not in ("ok", "unknown status")
    assert sw.swarm_status_string(-99) == "unknown status"


def test_workspace_bytes_and_config_validation(lib):
    ok = sw.StageConfig(256, 4, 1024, 1, 1, 4, 128, "f32")
    fwd = sw.swarm_stage_workspace_bytes(ok, False)
    bwd = sw.swarm_stage_workspace_bytes(ok, True)
    T, d, f = 512, 256, 1024
    assert fwd >= (7 * T * d + T * f) * 4 and fwd % 256 == 0
    assert bwd > fwd
    # more applications need more backward workspace, forward only the ping-pong buffers
    ok4 = sw.StageConfig(256, 4, 1024, 1, 4, 4, 128, "f32")
    assert sw.swarm_stage_workspace_bytes(ok4, True) > 2.5 * bwd
    for bad in (sw.StageConfig(250, 5, 1024, 1, 1, 4, 128, "f32"),      # d_model % 64
                sw.StageConfig(256, 8, 1024, 1, 1, 4, 128, "f32"),      # d_head 32
                sw.StageConfig(256, 4, 1000, 1, 1, 4, 128, "f32"),      # d_ffn % 64
                sw.StageConfig(256, 4, 1024, 0, 1, 4, 128, "f32"),
                sw.StageConfig(256, 4, 1024, 1, 1, 4, 0, "f32"),
                sw.StageConfig(256, 4, 1024, 1, 1, 4, 128, "f32", ln_eps=0.0)):
        assert sw.swarm_stage_workspace_bytes(bad, False) == 0
        assert sw.swarm_stage_workspace_bytes(bad, True) == 0


def test_null_and_shape_errors_without_gpu(lib):
    cfg = sw.StageConfig(256, 4, 1024, 1, 1, 4, 128, "f32")
    blocks = (binding._BlockPtrs * 1)()
    # null tensors
    assert lib.swarm_stage_forward(C.byref(cfg.c), blocks, None, None, None, 0, None) == -1
    assert lib.swarm_stage_backward(C.byref(cfg.c), blocks, None, None, None, blocks, None, 0, None) == -1
    # non-null tensors but null parameter pointers
    assert lib.swarm_stage_forward(C.byref(cfg.c), blocks, 4096, 8192, 256 * 40, 1 << 30, None) == -1
    bad = sw.StageConfig(256, 4, 1024, 1, 1, 4, 128, "f32")
    bad.c.dtype = 9
    assert lib.swarm_stage_forward(C.byref(bad.c), blocks, 4096, 8192, 256 * 40, 1 << 30, None) == -3
    # codec: wrong block, wrong dtype, null, misaligned; empty is fine
    assert lib.swarm_codec_encode(4096, 1, 128, 32, 8192, 12288, None) == -2
    assert lib.swarm_codec_encode(4096, 7, 128, 64, 8192, 12288, None) == -3
    assert lib.swarm_codec_encode(None, 1, 128, 64, 8192, 12288, None) == -1
    assert lib.swarm_codec_encode(4098, 1, 128, 64, 8192, 12288, None) == -2
    assert lib.swarm_codec_encode(None, 1, 0, 64, None, None, None) == 0
    assert lib.swarm_codec_decode(None, None, 0, 64, None, 1, None) == 0
    assert lib.swarm_codec_decode(None, 4096, 64, 64, 8192, 1, None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setenv("SWARM_STAGE_LIB", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()
    monkeypatch.delenv("SWARM_STAGE_LIB")
    monkeypatch.setattr(binding, "_lib", None)


def test_boundary_layer_validation_without_gpu(lib):
    ok = sw.BoundaryConfig(256, 128, "bottleneck", 64, "f32")
    assert sw.swarm_boundary_workspace_bytes(ok, False, False) > 0
    assert sw.swarm_boundary_workspace_bytes(ok, False, True) > sw.swarm_boundary_workspace_bytes(ok, False, False)
    assert sw.swarm_boundary_workspace_bytes(ok, True, True) > 0
    for bad in (sw.BoundaryConfig(250, 128, "bottleneck", 64, "f32"),     # d_model % 64
                sw.BoundaryConfig(256, 100, "bottleneck", 64, "f32"),     # d_comp % 32
                sw.BoundaryConfig(256, 512, "bottleneck", 64, "f32"),     # c > m
                sw.BoundaryConfig(256, 96, "maxout", 64, "f32"),          # m % c for maxout
                sw.BoundaryConfig(256, 128, "bottleneck", 0, "f32"),
                sw.BoundaryConfig(256, 128, "bottleneck", 64, "f32", ln_eps=0.0)):
        assert sw.swarm_boundary_workspace_bytes(bad, False, False) == 0
    # null pointers are refused before anything touches a device
    null3 = binding._Ptrs3(None, None, None)
    st = lib.swarm_compress_forward(C.byref(ok.c), C.byref(null3), None, None, None, 0, None)
    assert st == -1
    st = lib.swarm_decompress_backward(C.byref(ok.c), C.byref(null3), None, None, None, C.byref(null3), None, 0, None)
    assert st == -1


def test_head_validation_without_gpu(lib):
    ok = sw.HeadConfig(256, 1000, 1024, 64, "f32")
    assert sw.swarm_head_workspace_bytes(ok, True) > sw.swarm_head_workspace_bytes(ok, False) > 0
    for bad in (sw.HeadConfig(250, 1000, 1024, 64, "f32"),      # d_model % 64
                sw.HeadConfig(256, 1000, 999, 64, "f32"),       # fewer rows than tokens in the vocabulary
                sw.HeadConfig(256, 1000, 1004, 64, "f32"),      # rows % 8
                sw.HeadConfig(256, 0, 1024, 64, "f32"),
                sw.HeadConfig(256, 1000, 1024, 0, "f32")):
        assert sw.swarm_head_workspace_bytes(bad, False) == 0
    null3 = binding._Ptrs3(None, None, None)
    assert lib.swarm_head_loss(C.byref(ok.c), C.byref(null3), None, None, None, None, None, 0, None) == -1
    assert lib.swarm_embedding_forward(None, None, 0, 4, 10, 64, None, None) == -1
    # shape errors come before any launch: the pointers below are never dereferenced
    dummy = C.c_void_p(256)
    assert lib.swarm_embedding_backward(dummy, dummy, 1, 70000, 10, 64, dummy, None) == -2   # T > 65536
    assert lib.swarm_embedding_forward(dummy, dummy, 1, 4, 10, 60, dummy, None) == -2        # d % 8


def test_lamb_validation_without_gpu(lib):
    assert sw.swarm_lamb_workspace_bytes(0) == 0
    assert sw.swarm_lamb_workspace_bytes(1000) >= 4000
    cfg = binding._LambConfig(1e-3, 0.9, 0.95, 1e-6, 0.01, 1.0, 1)
    assert lib.swarm_lamb_step(C.byref(cfg), 16, None, None, 0, None, None, None, None, None, 0, None) == -1
    dummy = C.c_void_p(256)
    bad = binding._LambConfig(1e-3, 0.9, 0.95, 1e-6, 0.01, 1.0, 0)                      # step 0
    assert lib.swarm_lamb_step(C.byref(bad), 16, dummy, None, 0, dummy, dummy, dummy, None, dummy, 1 << 20, None) == -2
    assert lib.swarm_lamb_step(C.byref(cfg), 16, dummy, None, 0, dummy, dummy, dummy, None, dummy, 8, None) == -4


def test_codec_s16_validation_without_gpu(lib):
    dummy = C.c_void_p(256)
    for fn in (lib.swarm_codec_encode_s16, lib.swarm_codec_decode_s16):
        fn.restype = C.c_int
    enc = lambda *a: lib.swarm_codec_encode_s16(*a)
    assert enc(dummy, 1, C.c_size_t(0), 64, dummy, dummy, None) == 0                 # empty: no-op
    assert enc(dummy, 1, C.c_size_t(64), 32, dummy, dummy, None) == -2               # block must be 64
    assert enc(dummy, 7, C.c_size_t(64), 64, dummy, dummy, None) == -3               # dtype
    assert enc(None, 1, C.c_size_t(64), 64, dummy, dummy, None) == -1
    assert enc(dummy, 1, C.c_size_t(64), 64, dummy, C.c_void_p(257), None) == -2     # scales 2-byte aligned
    assert lib.swarm_codec_decode_s16(dummy, None, C.c_size_t(64), 64, dummy, 1, None) == -1


def test_headers_are_c99_and_binding_structs_match_their_layout(tmp_path):
    """The ABI headers compile as plain C99 (and as C++), and every struct the binding mirrors with ctypes has the
    size and field offsets the C compiler gives it."""
    import ctypes
    import shutil
    import subprocess
    from paper_2301_11913_amd import binding as b
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    inc = os.path.join(ROOT, "include")
    structs = {
        "swarm_stage_config": (b._Config, "swarm_stage.h"),
        "swarm_block_params": (b._BlockPtrs, "swarm_stage.h"),
        "swarm_block_grads": (b._BlockPtrs, "swarm_stage.h"),
        "swarm_boundary_config": (b._BoundaryConfig, "swarm_boundary.h"),
        "swarm_compress_params": (b._Ptrs3, "swarm_boundary.h"),
        "swarm_decompress_grads": (b._Ptrs3, "swarm_boundary.h"),
        "swarm_head_config": (b._HeadConfig, "swarm_head.h"),
        "swarm_head_params": (b._Ptrs3, "swarm_head.h"),
        "swarm_lamb_config": (b._LambConfig, "swarm_optim.h"),
    }
    c_fields = {"swarm_compress_params": ["ln_g", "ln_b", "w_c"], "swarm_decompress_grads": ["ln_g", "ln_b", "w_d"],
                "swarm_head_params": ["ln_g", "ln_b", "w_vocab"]}
    lines = ['#include <stdio.h>', '#include <stddef.h>']
    lines += ['#include "%s"' % h for h in sorted({h for _, h in structs.values()})]
    lines.append("int main(void) {")
    for name, (ct, _) in structs.items():
        names = c_fields.get(name, [f for f, _ in ct._fields_])
        lines.append('  printf("%s %%zu", sizeof(%s));' % (name, name))
        for f in names:
            lines.append('  printf(" %%zu", offsetof(%s, %s));' % (name, f))
        lines.append('  printf("\\n");')
    lines.append("  return 0; }")
    src = tmp_path / "probe.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = {l.split()[0]: [int(x) for x in l.split()[1:]] for l in out if l.strip()}
    for name, (ct, _) in structs.items():
        want = [ctypes.sizeof(ct)] + [getattr(ct, f).offset for f, _ in ct._fields_]
        assert seen[name] == want, (name, seen[name], want)
    if shutil.which("g++"):
        cxx = tmp_path / "probe.cpp"
        cxx.write_text("\n".join('#include "%s"' % h for h in sorted(os.listdir(inc)) if h.endswith(".h")) + "\nint main() { return 0; }\n")
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cxx)], check=True)


def test_lamb_static_validation_without_gpu(lib):
    """The entry point without workspace rejects what the host can see before it looks up its device scratch."""
    cfg = binding._LambConfig(1e-3, 0.9, 0.95, 1e-6, 0.01, 1.0, 1)
    f = lib.swarm_lamb_step_static
    assert f(C.byref(cfg), 1024, None, None, 0, 4096, 8192, 12288, None, None) == -1             # null master weights
    assert f(C.byref(cfg), 0, 4096, None, 0, 8192, 12288, 16384, None, None) == -2                # empty tensor
    assert f(C.byref(cfg), 1024, 4100, None, 0, 8192, 12288, 16384, None, None) == -2             # misaligned
    assert f(C.byref(cfg), sw.SWARM_LAMB_STATIC_MAX_ELEMS + 1, 4096, None, 0, 8192, 12288, 16384, None, None) == -4
    bad = binding._LambConfig(1e-3, 1.5, 0.95, 1e-6, 0.01, 1.0, 1)
    assert f(C.byref(bad), 1024, 4096, None, 0, 8192, 12288, 16384, None, None) == -2
