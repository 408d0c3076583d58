"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every
symbol the header declares, and its pure-host entry points behave."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2106_11257_amd as btard
from paper_2106_11257_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "btard.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(btard_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = btard.load_library()
    names = declared_functions()
    assert {"btard_centered_clip", "btard_verify_projections", "btard_split_offsets",
            "btard_workspace_bytes", "btard_cc_begin", "btard_cc_iterate",
            "btard_cc_finish"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None
        assert hasattr(btard, name), f"python binding lacks {name}"


@pytest.mark.parametrize("d,parts", [(10, 3), (0, 4), (7, 8), (11173962, 16), (1315758080, 16),
                                     (17683968, 64), (1000003, 7)])
def test_split_offsets_follow_the_paper_rule(d, parts):
    off = btard.split_offsets(d, parts)
    assert off == list(oracle.split(d, parts))          # two independent implementations
    sizes = np.diff(off)
    assert (sizes[: d % parts] == -(-d // parts)).all() and (sizes[d % parts:] == d // parts).all()


def test_split_offsets_rejects_bad_arguments():
    lib = btard.load_library()
    buf = (ctypes.c_int64 * 4)()
    assert lib.btard_split_offsets(-1, 3, buf) == -1
    assert lib.btard_split_offsets(5, 0, buf) == -1
    assert lib.btard_split_offsets(5, 3, None) == -1


def test_workspace_bytes():
    assert btard.workspace_bytes(0, 4) == 0
    assert btard.workspace_bytes(256, 4) == 0
    assert btard.workspace_bytes(16, 0) == 0
    a, b, c = (btard.workspace_bytes(16, 16), btard.workspace_bytes(64, 64),
               btard.workspace_bytes(255, 65535))
    assert 0 < a < b < c < (1 << 31)
    assert a % 256 == 0 and b % 256 == 0


def test_status_strings():
    lib = btard.load_library()
    assert lib.btard_status_string(0) == b"BTARD_OK"
    assert lib.btard_status_string(-1) == b"BTARD_ERR_INVALID_ARG"
    assert lib.btard_status_string(-2) == b"BTARD_ERR_WORKSPACE"
    assert lib.btard_status_string(-3) == b"BTARD_ERR_DEVICE"


def test_argument_errors_are_caught_on_the_host_before_any_gpu_call():
    lib = btard.load_library()
    off = (ctypes.c_int64 * 3)(0, 4, 8)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    ws = ctypes.c_void_p(0x10000)
    big = 1 << 30

    def cc(g=fake, ld=8, n=2, d=8, o=off, parts=2, tau=1.0, eps=1e-6, m=5, v0=None, v=fake,
           iters=fake, wsp=ws, wsb=big, flags=0):
        return lib.btard_centered_clip(g, ld, n, d, o, parts, tau, eps, m, v0, v, iters, None,
                                       wsp, wsb, None, flags)

    assert cc(g=None) == -1
    assert cc(n=0) == -1 and cc(n=256) == -1
    assert cc(ld=7) == -1
    assert cc(d=9) == -1                       # offsets must end at d
    assert cc(parts=0) == -1
    assert cc(o=(ctypes.c_int64 * 3)(0, 9, 8)) == -1
    assert cc(o=(ctypes.c_int64 * 3)(1, 4, 8)) == -1
    assert cc(tau=0.0) == -1 and cc(tau=float("nan")) == -1
    assert cc(eps=-1.0) == -1 and cc(m=-1) == -1
    assert cc(flags=16) == -1 and cc(flags=31) == -1
    assert cc(wsp=None) == -2
    assert cc(wsp=ctypes.c_void_p(0x10001)) == -2      # misaligned
    assert cc(wsb=16) == -2
    assert cc(v=None) == -1 and cc(iters=None) == -1
    assert cc(v0=fake, v=fake) == -1                   # v must not overlap v0

    def gm(g=fake, n=2, nu=1e-6, eps=1e-6, m=5, v=fake, wsb=big):
        return lib.btard_geometric_median(g, 8, n, 8, off, 2, nu, eps, m, None, v, fake, None, ws,
                                          wsb, None)

    assert gm(g=None) == -1 and gm(n=0) == -1 and gm(nu=0.0) == -1 and gm(m=-1) == -1
    assert gm(v=None) == -1 and gm(wsb=16) == -2

    def cm(g=fake, ld=8, n=2, d=8, v=fake):
        return lib.btard_coordinate_median(g, ld, n, d, v, None)

    assert cm(g=None) == -1 and cm(v=None) == -1 and cm(n=0) == -1 and cm(n=256) == -1
    assert cm(ld=7) == -1 and cm(d=-1) == -1
    assert cm(g=None, v=None, d=0, ld=0) == 0          # nothing to do

    def v12(a=fake, n=2, parts=2, rtol=1e-6, atol=0.0, out=fake):
        return lib.btard_verification12(a, fake, fake, fake, n, parts, rtol, atol, out, fake, fake,
                                        None)

    assert v12(a=None) == -1 and v12(out=None) == -1 and v12(n=0) == -1 and v12(parts=0) == -1
    assert v12(rtol=-1.0) == -1 and v12(atol=float("nan")) == -1

    def vp(g=fake, v=fake, norms=fake, tau=1.0, delta=None, ldd=0, wsb=big):
        return lib.btard_verify_projections(g, 8, 2, 8, off, 2, v, tau, 1, norms, fake, fake, None,
                                            delta, ldd, ws, wsb, None, 0)

    assert vp(g=None) == -1 and vp(v=None) == -1 and vp(norms=None) == -1
    assert vp(tau=-1.0) == -1
    assert vp(delta=ctypes.c_void_p(0x2000000), ldd=4) == -1
    assert vp(wsb=8) == -2

    def vpp(g=fake, v=fake, lam=1.0, fac=None, tau=1.0, wsb=big):
        return lib.btard_verify_projections_preclipped(g, 8, 2, 8, off, 2, v, lam, fac, tau, 1, fake,
                                                       fake, fake, None, None, 0, None, ws, wsb,
                                                       None, 0)

    assert vpp(g=None) == -1 and vpp(v=None) == -1 and vpp(tau=0.0) == -1
    # neither factors nor a usable radius
    assert vpp(lam=0.0) == -1 and vpp(lam=float("inf")) == -1 and vpp(lam=float("nan")) == -1
    assert vpp(wsb=8) == -2 and vpp(lam=0.0, fac=fake, wsb=8) == -2


    def plain(g=fake, ld=8, n=2, d=8, v=None, blocks=4):
        return lib.btard_debug_plain_stream(g, ld, n, d, v, blocks, None)

    assert plain(g=None) == -1 and plain(n=0) == -1 and plain(blocks=0) == -1
    assert plain(d=-1) == -1 and plain(ld=7, d=8) == -1 and plain(n=256) == -1
    assert plain(blocks=(1 << 20) + 1) == -1
    assert plain(d=0, ld=0) == 0                                 # nothing to do


def test_binding_constants_match_the_header():
    """The flag and limit values of the Python binding are those of include/btard.h."""
    import re
    from paper_2106_11257_amd import binding
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                               "include", "btard.h")).read()
    defines = dict(re.findall(r"#define\s+(BTARD_[A-Z_]+)\s+(\d+)u?\b", header))
    flags = [k for k in defines if k.startswith("BTARD_FLAG_")]
    assert len(flags) >= 5
    for name in flags:
        assert getattr(binding, name) == int(defines[name]), name
    # the flags are distinct bits
    bits = [int(defines[k]) for k in flags if int(defines[k]) != 0]
    assert len(set(bits)) == len(bits) and all(b & (b - 1) == 0 for b in bits)


def test_header_is_plain_c_and_a_c_program_calls_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and as C++11 without warnings,
    and a C program linked against the library calls a host entry point."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "caller.c"
    src.write_text(
        '#include <stdio.h>\n#include "btard.h"\n'
        "int main(void) {\n"
        "    int64_t off[4];\n"
        "    if (btard_split_offsets(10, 3, off) != 0) return 1;\n"
        '    printf("%lld %lld %lld %lld\\n", (long long)off[0], (long long)off[1],\n'
        "           (long long)off[2], (long long)off[3]);\n"
        "    return btard_split_offsets(-1, 3, off) == -1 ? 0 : 2;\n"
        "}\n")
    flags = ["-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc]
    subprocess.run(["gcc", "-std=c99", *flags, "-fsyntax-only", str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", *flags, "-fsyntax-only", "-x", "c++", str(src)], check=True)
    btard.load_library()
    libdir = os.path.dirname(binding._LIB_PATH)
    exe = tmp_path / "caller"
    subprocess.run(["gcc", "-std=c99", *flags, str(src), "-o", str(exe), "-L", libdir, "-lbtard",
                    f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(x) for x in out] == [0, 4, 7, 10]
