"""CPU-side checks of the C-ABI library: it loads, exports every declared entry
point, and its host-only functions (record layout, buffer sizes, argument
validation) agree with the oracle.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from oracle import mixkvq_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def M():
    import paper_2512_19206_amd as M
    if not os.path.exists(M.LIB_PATH):
        from paper_2512_19206_amd.build import build_library
        build_library()
    return M


def _declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(mixkvq_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol(M):
    lib = M.load_library()
    declared = _declared_symbols()
    assert declared, "no declarations found"
    assert declared == set(M.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


CONFIGS = [
    dict(B=1, Hq=1, Hkv=1, D=128, T_max=1024, Gk=32, Gv=32, R=32, k4=8, k16=0),
    dict(B=8, Hq=28, Hkv=4, D=128, T_max=32768, Gk=128, Gv=128, R=128, k4=16, k16=0),
    dict(B=64, Hq=40, Hkv=8, D=128, T_max=32768, Gk=128, Gv=128, R=128, k4=0, k16=12),
    dict(B=2, Hq=8, Hkv=2, D=128, T_max=256, Gk=16, Gv=16, R=64, k4=8, k16=4),
    dict(B=1, Hq=2, Hkv=2, D=128, T_max=128, Gk=64, Gv=64, R=128, k4=0, k16=0),
    dict(B=2, Hq=14, Hkv=2, D=128, T_max=512, Gk=128, Gv=128, R=128, k4=16, k16=8, policy=1, tau16=1.44, tau4=0.79),
    dict(B=2, Hq=14, Hkv=2, D=128, T_max=512, Gk=32, Gv=32, R=128, k4=16, k16=0),
    dict(B=2, Hq=14, Hkv=2, D=128, T_max=512, Gk=32, Gv=32, R=128, k4=16, k16=0, sink=32),
    dict(B=1, Hq=5, Hkv=1, D=128, T_max=64, Gk=32, Gv=32, R=32, k4=8, k16=4, policy=1, tau16=0.0, tau4=float("inf")),
    dict(B=2, Hq=14, Hkv=2, D=128, T_max=1024, Gk=64, Gv=128, R=256, k4=16, k16=0, sink=32),
    dict(B=2, Hq=14, Hkv=2, D=128, T_max=960, Gk=32, Gv=32, R=96, k4=16, k16=0),
    dict(B=1, Hq=2, Hkv=1, D=128, T_max=192, Gk=48, Gv=64, R=96, k4=8, k16=0),
]


@pytest.mark.parametrize("kw", CONFIGS)
def test_record_layout_matches_oracle(M, kw):
    lay = M.block_layout(M.make_config(**kw))
    ref = O.block_layout(O.OracleConfig(**kw))
    for name, _ in lay._fields_:
        assert getattr(lay, name) == getattr(ref, name), name


@pytest.mark.parametrize("kw", CONFIGS)
def test_buffer_sizes(M, kw):
    cfg = M.make_config(**kw)
    sz, lay = M.cache_sizes(cfg), M.block_layout(cfg)
    P = kw["B"] * kw["Hkv"]
    assert sz.blocks >= P * (kw["T_max"] // O.rec_tokens(O.OracleConfig(**kw))) * lay.rec_bytes
    assert sz.res_k >= P * (kw["R"] + kw.get("sink", 0)) * 128 * 2 and sz.res_v == sz.res_k
    assert sz.qacc >= P * 129 * 8
    assert sz.workspace >= P * 128 * 16
    for f in ("blocks", "res_k", "res_v", "qacc", "workspace"):
        assert getattr(sz, f) % 256 == 0


@pytest.mark.parametrize("bad", [
    dict(D=64), dict(Hq=3, Hkv=2), dict(Hq=18, Hkv=2), dict(R=24), dict(R=192, T_max=384), dict(R=256, T_max=256, Gk=256), dict(Gk=48),
    dict(Gv=24), dict(k4=4), dict(k16=2), dict(k4=64, k16=64), dict(T_max=100), dict(flush_mode=2),
    dict(score_mode=-1), dict(B=0), dict(policy=2), dict(policy=1, tau16=-0.5, tau4=1.0),
    dict(policy=1, tau16=1.0, tau4=float("nan")), dict(sink=16), dict(sink=160), dict(sink=-32),
])
def test_bad_configurations_are_rejected(M, bad):
    kw = dict(CONFIGS[1])
    kw.update(bad)
    cfg = M.make_config(**kw)
    lay = M.BlockLayout()
    assert M.load_library().mixkvq_block_layout(C.byref(cfg), C.byref(lay)) == -1
    sz = M.Sizes()
    assert M.load_library().mixkvq_cache_sizes(C.byref(cfg), C.byref(sz)) == -1


def test_null_arguments_and_error_strings(M):
    lib = M.load_library()
    assert lib.mixkvq_block_layout(None, None) == -1
    assert lib.mixkvq_cache_state(None, None, None, None) == -1
    assert lib.mixkvq_decode_attention(None, None, None, None, 0.0, 0, None) == -1
    assert lib.mixkvq_decode_path(None) == -1
    assert lib.mixkvq_quantize_append(None, None, None, 1, None, None, None) == -1
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(lib.mixkvq_strerror(code)) > 0
    # cache_create rejects NULL and misaligned device pointers before touching the device
    cfg = M.make_config(**CONFIGS[0])
    h = C.c_void_p()
    bufs = M.binding.Buffers(0, 0, 0, 0, 0)
    assert lib.mixkvq_cache_create(C.byref(cfg), C.byref(bufs), C.byref(h)) == -1
    bufs = M.binding.Buffers(256, 256, 256, 256, 260)
    assert lib.mixkvq_cache_create(C.byref(cfg), C.byref(bufs), C.byref(h)) == -1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the public header must compile as C99 on its own, and a C program that fills the
    structs sees the sizes the Python binding assumes."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi.c"
    src.write_text('#include "mixkvq.h"\n#include <stdio.h>\n'
                   'int main(void) { mixkvq_config c = {0}; mixkvq_block_layout_t l; (void)c; (void)l;\n'
                   '  printf("%zu %zu %zu %zu\\n", sizeof(mixkvq_config), sizeof(mixkvq_block_layout_t),\n'
                   '         sizeof(mixkvq_sizes), sizeof(mixkvq_buffers)); return 0; }\n')
    exe = tmp_path / "abi"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe)], check=True)
    sizes = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    import paper_2512_19206_amd.binding as Bd
    assert sizes == [C.sizeof(Bd.Config), C.sizeof(Bd.BlockLayout), C.sizeof(Bd.Sizes), C.sizeof(Bd.Buffers)]


def test_host_state_machine_under_address_and_undefined_behaviour_sanitizers(M, tmp_path):
    """csrc/api.hip (configuration checks, layout, handle, token-count state machine, error paths) compiled with
    -fsanitize=address and -fsanitize=undefined on the HOST side, linked with the regular kernel objects and driven by
    tests/host_shim_driver.c.  Host functions only: no kernel runs (without a GPU the launches fail inside HIP, and
    the driver checks that such a failure leaves the token counts unchanged)."""
    import subprocess
    from paper_2512_19206_amd import build as B
    objs = [os.path.join(B.OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in B.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in objs):
        B.build_library()
    hipcc = B.hipcc_path()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    api_o = str(tmp_path / "api_san.o")
    drv_o = str(tmp_path / "driver.o")
    exe = str(tmp_path / "host_shim_driver")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", B.CSRC]
    run = lambda cmd: subprocess.run(cmd, capture_output=True, text=True)
    r = run([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC"] + san + inc +
            ["-c", os.path.join(B.CSRC, "api.hip"), "-o", api_o])
    assert r.returncode == 0, r.stdout + r.stderr
    r = run(["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Werror", "-fsanitize=address", "-fsanitize=undefined",
             "-fno-sanitize-recover=undefined"] + inc + ["-c", os.path.join(ROOT, "tests", "host_shim_driver.c"), "-o", drv_o])
    assert r.returncode == 0, r.stdout + r.stderr
    r = run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
             drv_o, api_o] + objs + ["-o", exe])
    assert r.returncode == 0, r.stdout + r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host shim driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
