"""The C-ABI library: it loads, exports every symbol the header declares, and its
host-only entry points behave (no GPU compute here)."""

import os
import re

import numpy as np
import pytest

from oracle import curdkv_oracle as orc
from paper_2509_15038_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "curdkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(curdkv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "curdkv_scores" in names and "curdkv_select" in names and "curdkv_compact" in names
    L = B.lib()
    for nm in names:
        assert hasattr(L, nm), nm
    assert sorted(B.EXPORTS) == names


def test_strerror():
    assert B.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert B.strerror(code)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("r", [20, 32, 64, 128])
def test_host_sketch_matches_oracle_bitwise(dtype, r):
    # two independent implementations of the same counter-based generator
    cfg = B.make_config(3, 8, 4, 128, r, dtype, 1024, 0xC0DE0003)
    for (l, h) in [(0, 0), (1, 5), (2, 7)]:
        got = B.curdkv_sketch_host(cfg, l, h)
        want = orc.sketch(0xC0DE0003, l, h, 8, 128, r, dtype)
        assert np.array_equal(got.astype(np.float64), want)


def test_config_validation_on_host():
    G = np.empty((128, 64), dtype=np.float32)
    import ctypes as C
    def rc(**kw):
        base = dict(layers=1, kv_heads=1, group_size=1, head_dim=128, sketch_dim=64, dtype="bf16",
                    max_tokens=16, seed=1)
        base.update(kw)
        cfg = B.make_config(**base)
        return B.lib().curdkv_sketch_host(C.byref(cfg), 0, 0, G.ctypes.data)
    assert rc() == B.OK
    assert rc(head_dim=64) == B.ERR_UNSUPPORTED
    assert rc(sketch_dim=129) == B.ERR_UNSUPPORTED
    assert rc(sketch_dim=0) == B.ERR_INVALID_ARG
    assert rc(dtype=7) == B.ERR_UNSUPPORTED
    assert rc(layers=0) == B.ERR_INVALID_ARG
    assert rc(max_tokens=0) == B.ERR_INVALID_ARG
    cfg = B.make_config(1, 1, 1, 128, 64, "bf16", 16, 1)
    assert B.lib().curdkv_sketch_host(C.byref(cfg), 1, 0, G.ctypes.data) == B.ERR_INVALID_ARG
    assert B.lib().curdkv_sketch_host(C.byref(cfg), 0, 0, None) == B.ERR_INVALID_ARG
    assert B.lib().curdkv_sketch_host(None, 0, 0, G.ctypes.data) == B.ERR_INVALID_ARG


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and a C program must
    # be able to link against the library and call its host-only entry points
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_curdkv.c"
    src.write_text(r'''
#include "curdkv.h"
#include <stdio.h>
#include <string.h>
int main(void) {
    curdkv_config cfg;
    static float G[128 * 64];
    unsigned bits;
    int i;
    memset(&cfg, 0, sizeof cfg);
    cfg.layers = 3; cfg.kv_heads = 8; cfg.group_size = 4; cfg.head_dim = 128; cfg.sketch_dim = 64;
    cfg.dtype = CURDKV_DTYPE_BF16; cfg.max_tokens = 1024; cfg.seed = 0xC0DE0003u;
    if (curdkv_sketch_host(&cfg, 2, 7, G) != CURDKV_OK) return 1;
    for (i = 0; i < 6; ++i) { memcpy(&bits, &G[i * 1000], 4); printf("%08x\n", bits); }
    cfg.head_dim = 96;
    printf("%d %s\n", curdkv_sketch_host(&cfg, 0, 0, G), curdkv_strerror(CURDKV_ERR_UNSUPPORTED));
    return 0;
}
''')
    pkg = os.path.join(ROOT, "paper_2509_15038_amd")
    exe = tmp_path / "use_curdkv"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", pkg, "-lcurdkv", f"-Wl,-rpath,{pkg}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    want = orc.sketch(0xC0DE0003, 2, 7, 8, 128, 64, "bf16").astype(np.float32).reshape(-1)
    for i in range(6):
        assert int(out[i], 16) == int(want[i * 1000].view(np.uint32)), i
    assert out[6].startswith(f"{B.ERR_UNSUPPORTED} unsupported")


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    # no CPU fallback: without the built library every use of the binding raises
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libcurdkv.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()
    with pytest.raises(RuntimeError):
        B.Context(1, 1, 1, 128, 32, "bf16", 16, 1)
    with pytest.raises(RuntimeError):
        B.strerror(0)


_SAN_HARNESS = r"""
#include <cstdio>
#include <cstring>
#include <vector>
#include "curdkv_internal.h"
using namespace curdkv;
int main() {
    // for every (dtype, r): G of a few groups, packed into a buffer of exactly the packed size
    // (the sanitizer puts red zones around it); prints a checksum of the values and of the packing
    const int rs[] = {1, 20, 32, 33, 64, 100, 128};
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int r : rs) {
            curdkv_config cfg{};
            cfg.layers = 3; cfg.kv_heads = 8; cfg.group_size = 4; cfg.head_dim = 128; cfg.sketch_dim = r;
            cfg.dtype = dtype; cfg.max_tokens = 64; cfg.seed = 0xC0DE0003ull;
            const int cbs = r <= 32 ? 1 : (r <= 64 ? 2 : 4);
            std::vector<float> G((size_t)128 * r);
            std::vector<unsigned char> packed(packed_elems(cbs) * (dtype == CURDKV_DTYPE_BF16 ? 2 : 4));
            for (int l : {0, 2}) for (int h : {0, 7}) {
                sketch_values(cfg, l, h, G.data());
                pack_sketch(cfg, cbs, G.data(), packed.data());
                unsigned long long a = 1469598103934665603ull, b = a;
                for (float g : G) { unsigned u; std::memcpy(&u, &g, 4); a = (a ^ u) * 1099511628211ull; }
                for (unsigned char c : packed) b = (b ^ c) * 1099511628211ull;
                std::printf("%d %d %d %d %016llx %016llx\n", dtype, r, l, h, a, b);
            }
        }
    return 0;
}
"""


def _fnv(words, width):
    a = 1469598103934665603
    for w in words:
        a = ((a ^ int(w)) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return a


def test_sketch_host_code_under_address_and_ub_sanitizers(tmp_path):
    # the host code that generates and packs the sketches, built for the CPU alone with
    # AddressSanitizer and UBSan: no out-of-bounds access, no undefined arithmetic, and the
    # values (against the oracle) and the operand packing (against the layout the kernels'
    # comments state, written out here independently) are what they should be
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None or not os.path.isdir("/opt/rocm/include"):
        pytest.skip("needs g++ and the HIP headers")
    src = tmp_path / "harness.cpp"
    src.write_text(_SAN_HARNESS)
    exe = tmp_path / "harness"
    csrc = os.path.join(ROOT, "paper_2509_15038_amd", "csrc")
    subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-static-libubsan",
                    "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", csrc, "-I", "/opt/rocm/include",
                    os.path.join(csrc, "sketch_host.cpp"), str(src), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert p.returncode == 0, p.stderr[-3000:]
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr[-3000:]
    lines = [ln.split() for ln in p.stdout.strip().split("\n")]
    assert len(lines) == 2 * 7 * 4
    for dt, r, l, h, ha, hb in lines:
        dt, r, l, h = int(dt), int(r), int(l), int(h)
        dtype = "bf16" if dt == 1 else "fp32"
        G = orc.sketch(0xC0DE0003, l, h, 8, 128, r, dtype).astype(np.float32)
        assert int(ha, 16) == _fnv(G.reshape(-1).view(np.uint32), 4), (dtype, r, l, h)
        cbs = 1 if r <= 32 else (2 if r <= 64 else 4)
        Gp = np.zeros((128, 32 * cbs), dtype=np.float32)
        Gp[:, :r] = G
        if dtype == "bf16":
            # [16-column block][step 0..3][lane][8 values]: rows s*32 + (lane//16)*8 + e, column cb*16 + lane%16
            bits = orc.f32_to_bf16_bits(Gp)
            out = np.empty((2 * cbs, 4, 64, 8), dtype=np.uint16)
            for cb in range(2 * cbs):
                for st in range(4):
                    for lane in range(64):
                        rows = st * 32 + (lane // 16) * 8 + np.arange(8)
                        out[cb, st, lane] = bits[rows, cb * 16 + lane % 16]
        else:
            # [16-column block][step 0..7][lane][4 values]: rows (s*4 + lane//16)*4 + e, column cb*16 + lane%16
            out = np.empty((2 * cbs, 8, 64, 4), dtype=np.float32)
            for cb in range(2 * cbs):
                for st in range(8):
                    for lane in range(64):
                        rows = (st * 4 + lane // 16) * 4 + np.arange(4)
                        out[cb, st, lane] = Gp[rows, cb * 16 + lane % 16]
        assert int(hb, 16) == _fnv(out.reshape(-1).view(np.uint8), 1), ("packing", dtype, r, l, h)
