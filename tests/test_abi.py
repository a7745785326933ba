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
