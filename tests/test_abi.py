"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, sizes the weight blob like the generator, and rejects bad
configurations and policies before touching a device.  No compute calls."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1906_11024_amd import binding as sb
from paper_1906_11024_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sb.LIB_PATH):
        from paper_1906_11024_amd import build
        build.build(verbose=False)
    return sb.lib()


def test_library_is_built_from_the_current_sources(lib):
    """the binary that the GPU tests and the benchmark will load is the one csrc/ describes"""
    st = sb.lib_state()
    assert st["built_from"], "no build record next to libsan.so: run python -m paper_1906_11024_amd.build"
    assert not st["stale"], st


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "san.h")).read()
    declared = re.findall(r"SAN_API\s+[\w\s\*]+?\b(san_\w+)\s*\(", hdr)
    assert len(declared) >= 10
    assert sorted(declared) == sorted(sb.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_config_struct_matches_header(lib):
    hdr = open(os.path.join(ROOT, "include", "san.h")).read()
    body = hdr[hdr.index("typedef struct {"):hdr.index("} san_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in re.findall(r"(?:int32_t|float)\s+([^;]+);", body):
        names += [n.strip() for n in decl.split(",")]
    assert names == [f[0] for f in sb.SanConfig._fields_]
    assert C.sizeof(sb.SanConfig) == 4 * len(names)


@pytest.mark.parametrize("name", list(wl.CONFIGS))
def test_weight_bytes_matches_generator(lib, name):
    cfg = wl.get_config(name)
    n = sum(int(np.prod(s)) for _, s, _ in wl.tensor_specs(cfg))
    assert sb.weight_bytes(sb.make_config(cfg)) == n * (2 if cfg["dtype"] == "bf16" else 4)


def _init(lib, sc, self_pi, ctx_pi, nbytes=None, enc_pi=()):
    nbytes = sb.weight_bytes(sc) if nbytes is None else nbytes
    blob = np.zeros(max(nbytes, 4), dtype=np.uint8)
    sp = (C.c_int32 * max(1, len(self_pi)))(*self_pi)
    ep = (C.c_int32 * max(1, len(ctx_pi)))(*ctx_pi)
    pol = sb.SanPolicy(len(self_pi), C.cast(sp, C.POINTER(C.c_int32)), len(ctx_pi), C.cast(ep, C.POINTER(C.c_int32)),
                       len(enc_pi), C.cast((C.c_int32 * max(1, len(enc_pi)))(*enc_pi), C.POINTER(C.c_int32)) if enc_pi else None)
    h = C.c_void_p()
    rc = lib.san_init(C.byref(sc), blob.ctypes.data_as(C.c_void_p), nbytes, C.byref(pol), None, C.byref(h))
    assert rc != 0 and not h.value
    return rc, lib.san_last_error(None).decode()


@pytest.mark.parametrize("field,value", [("d_model", 100), ("d_model", 4096), ("n_heads", 3), ("n_heads", 64),
                                         ("d_ff", 100), ("vocab", 1001), ("beam", 0), ("beam", 33),
                                         ("dtype", 7), ("self_kind", 2), ("encdec_share", 5), ("max_tgt_len", 0),
                                         ("ln_eps", 0.0), ("n_dec_layers", 0), ("pad_id", -1), ("bos_id", 1000),
                                         ("eos_id", 1000), ("debug", 4), ("debug", -1)])
def test_bad_config_is_einval(lib, field, value):
    sc = sb.make_config(wl.get_config("tiny"))
    setattr(sc, field, value)
    assert sb.weight_bytes(sc) == 0
    rc, msg = _init(lib, sc, [2], [2], nbytes=16)
    assert rc == sb.SAN_EINVAL and msg


def test_blob_size_mismatch_is_einval(lib):
    sc = sb.make_config(wl.get_config("tiny"))
    rc, msg = _init(lib, sc, [2], [2], nbytes=sb.weight_bytes(sc) - 4)
    assert rc == sb.SAN_EINVAL and "bytes" in msg


@pytest.mark.parametrize("spi,cpi", [([1], [2]), ([2], [3]), ([0, 2], [2]), ([2], []), ([3], [2]), ([2], [1, -1, 2])])
def test_bad_policy_is_epolicy(lib, spi, cpi):
    """Sec. 3.3: the block sizes must sum to the number of layers."""
    sc = sb.make_config(wl.get_config("tiny"))
    rc, msg = _init(lib, sc, spi, cpi)
    assert rc == sb.SAN_EPOLICY and "policy" in msg


def test_bad_encoder_policy_is_epolicy(lib):
    sc = sb.make_config(wl.get_config("tiny"))
    for enc in ([1], [3], [2, 1], [0, 2]):
        rc, msg = _init(lib, sc, [2], [2], enc_pi=enc)
        assert rc == sb.SAN_EPOLICY and "encoder" in msg


def test_debug_needs_the_cache_and_null_handles(lib):
    sc = sb.make_config(wl.get_config("tiny"), use_cache=0, debug=1)
    rc, _ = _init(lib, sc, [2], [2], nbytes=16)
    assert rc == sb.SAN_EINVAL
    assert lib.san_step(None) == -1 and lib.san_device_bytes(None, 0) == 0
    assert lib.san_decode_step(None, None, None) == sb.SAN_EINVAL
    lib.san_free(None)


def test_fixed_scratch_is_a_dynamic_symbol_of_the_device_image(lib):
    """san_topk_noalloc's scratch array is found by name at run time (hipGetSymbolAddress), so
    the gfx950 image inside the library's object file must export it; a local symbol there
    aborts the process at san_init.  Reads the build's own object file with the LLVM tools."""
    import shutil
    import subprocess
    import tempfile
    obj = os.path.join(os.path.dirname(sb.LIB_PATH), "_build", "san.o")
    tools = "/opt/rocm/llvm/bin"
    need = [os.path.join(tools, t) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf")]
    if not os.path.exists(obj) or not all(os.path.exists(t) for t in need):
        pytest.skip("no object file of this build / no LLVM tools here")
    with tempfile.TemporaryDirectory() as td:
        fat, co = os.path.join(td, "fat.bin"), os.path.join(td, "dev.co")
        subprocess.run([need[0], f"--dump-section=.hip_fatbin={fat}", obj, os.path.join(td, "copy.o")], check=True)
        subprocess.run([need[1], "--unbundle", "--type=o", f"--input={fat}",
                        "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={co}"], check=True)
        out = subprocess.run([need[2], "--dyn-syms", co], check=True, capture_output=True, text=True).stdout
    rows = [l for l in out.splitlines() if "scratch" in l]
    assert rows and all("GLOBAL" in l and "OBJECT" in l for l in rows), out
    assert any(" 262144 " in l for l in rows), rows
