"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol declared in include/qtip.h, and turns bad arguments into error codes before
any GPU work is attempted."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def q():
    import paper_2406_11235_amd as q
    from paper_2406_11235_amd import build
    if build.is_stale():
        build.build()
    q.lib()
    return q


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qtip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qtip_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(q):
    names = declared_symbols()
    assert "qtip_decode_matvec" in names and "qtip_rht" in names and len(names) >= 9
    L = ctypes.CDLL(q.library_path())
    for name in names:
        assert hasattr(L, name), name
    from paper_2406_11235_amd import binding
    assert sorted(binding.EXPORTS) == names
    for name in names:
        assert hasattr(q, name), f"binding lacks {name}"


def test_version_matches_header(q):
    text = open(os.path.join(ROOT, "include", "qtip.h")).read()
    assert q.qtip_version() == int(re.search(r"#define QTIP_VERSION (\d+)", text).group(1))


def test_argument_errors_need_no_gpu(q):
    L = q.lib()
    buf = np.zeros(64, dtype=np.uint32)
    p = buf.ctypes.data                     # host memory: never dereferenced on these paths
    EINVAL, EUNSUP = -1, -2
    cases = [
        (L.qtip_decode_matvec(None, 16, 2, 1, 1, None, 16, 16, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 16, 2, 1, 1, None, 16, 16, None, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 16, 2, 1, 1, None, 24, 16, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 16, 2, 1, 1, None, 16, 0, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 14, 2, 1, 1, None, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p, 16, 5, 1, 1, None, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p, 16, 1, 1, 1, None, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p, 16, 2, 2, 1, None, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p, 16, 2, 1, 2, p, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p, 16, 2, 2, 2, None, 16, 16, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 16, 2, 1, 7, None, 16, 16, p, p, None), EUNSUP),
        (L.qtip_decode_matvec(p + 4, 16, 2, 1, 1, None, 16, 16, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 16, 2, 1, 1, None, 16, (1 << 28) + 16, p, p, None), EINVAL),   # above QTIP_MAX_N
        (L.qtip_decode_matvec(p, 16, 2, 1, 4, p, 32, 16, p, p, None), EUNSUP),       # the lookup-only code: L = 14
        (L.qtip_decode_matvec(p, 14, 2, 1, 4, None, 32, 16, p, p, None), EINVAL),   # needs its table
        (L.qtip_decode_matvec(p, 14, 2, 1, 4, p + 4, 32, 16, p, p, None), EINVAL),  # 16-byte aligned
        (L.qtip_decode_matvec(p, 14, 2, 1, 4, p, 16, 16, p, p, None), EINVAL),      # 32 x 8 blocks
        (L.qtip_decode_matvec(p, 14, 2, 1, 4, p, 32, 12, p, p, None), EINVAL),
        (L.qtip_decode_matvec(p, 14, 2, 2, 4, p, 32, 16, p, p, None), EUNSUP),
        (L.qtip_dequantize(p, 14, 5, 1, 4, p, 32, 16, p, None), EUNSUP),
        (L.qtip_decode_matmat(p, 16, 2, 1, 1, None, 16, 16, p, 0, None, p, None), EINVAL),
        (L.qtip_decode_matmat(p, 16, 2, 1, 1, None, 16, 16, p, 4, None, None, None), EINVAL),
        (L.qtip_dequantize(p, 16, 2, 1, 1, None, 16, 16, None, None), EINVAL),
        (L.qtip_dequantize(p, 16, 2, 1, 0, None, 16, 20, p, None), EINVAL),
        (L.qtip_decode_states(None, 4, 16, 1, 0, None, p, None), EINVAL),
        (L.qtip_decode_states(p, 4, 16, 2, 0, None, p, None), EUNSUP),
        (L.qtip_decode_states(p, -1, 16, 1, 0, None, p, None), EINVAL),
        (L.qtip_rht(None, p, 64, 64, 1, 0, p, None), EINVAL),
        (L.qtip_rht(p, p, 64, 48, 1, 0, p, None), EINVAL),
        (L.qtip_rht(p, p, 96, 64, 1, 0, p, None), EINVAL),
        (L.qtip_rht(p, p, 64, 64, 0, 0, p, None), EINVAL),
        (L.qtip_rht(p, p, 64, 64, 1, 2, p, None), EINVAL),
        (L.qtip_rht(p, p, 8, 8, 1, 0, p, None), EINVAL),
        (L.qtip_rht_f32(p, p, 64, 64, 1, 0, p, None), EINVAL),     # aliasing refused
        (L.qtip_rht_decode_matvec(p, 16, 2, 1, 1, None, 16, 64, None, p, 64, None, p, None, None), EINVAL),
        (L.qtip_rht_decode_matvec(p, 16, 2, 1, 1, None, 16, 64, p, p, 48, None, p, None, None), EINVAL),
        (L.qtip_rht_decode_matvec(p, 16, 2, 1, 1, None, 16, 96, p, p, 64, None, p, None, None), EINVAL),
        (L.qtip_rht_decode_matvec(p, 16, 2, 1, 1, None, 16, 16384, p, p, 64, None, p, None, None), EINVAL),
        (L.qtip_rht_decode_matvec(p, 16, 2, 1, 1, None, 8192, 64, p, p, 64, None, p, None, None), EINVAL),
        (L.qtip_rht_decode_matvec(p, 16, 7, 1, 1, None, 16, 64, p, p, 64, None, p, None, None), EUNSUP),
        (L.qtip_quantize(None, 16, 16, 16, 2, 1, 1, None, p, None), EINVAL),
        (L.qtip_quantize(p, 16, 16, 16, 2, 2, 2, None, p, None), EINVAL),
        (L.qtip_quantize(p, 16, 16, 16, 6, 1, 1, None, p, None), EUNSUP),
        (L.qtip_quantize(p, 16, 20, 16, 2, 1, 1, None, p, None), EINVAL),
        (L.qtip_quantize_gpu(None, 16, 16, 16, 2, 1, 1, None, p, None, 256, 1 << 21, None), EINVAL),
        (L.qtip_quantize_gpu(p, 16, 16, 16, 2, 1, 1, None, p, None, None, 1 << 21, None), EINVAL),
        (L.qtip_quantize_gpu(p, 16, 16, 16, 2, 1, 1, None, p, None, 256, 1000, None), EINVAL),
        (L.qtip_quantize_gpu(p, 16, 16, 16, 2, 1, 1, None, p, None, 260, 1 << 21, None), EINVAL),
        (L.qtip_quantize_gpu(p, 16, 16, 16, 2, 2, 2, None, p, None, 256, 1 << 21, None), EINVAL),
        (L.qtip_quantize_gpu(p, 16, 16, 12, 2, 1, 1, None, p, None, 256, 1 << 21, None), EUNSUP),
        (L.qtip_quantize_gpu(p, 16, 16, 16, 2, 2, 1, None, p, None, 256, 1 << 21, None), EUNSUP),
        (L.qtip_quantize_gpu(p, 16, 20, 16, 2, 1, 1, None, p, None, 256, 1 << 21, None), EINVAL),
    ]
    for i, (rc, want) in enumerate(cases):
        assert rc == want, (i, rc, want, q.qtip_last_error())
    assert "multiple of 16" in q.qtip_last_error()
    assert L.qtip_decode_states(p, 0, 16, 1, 0, None, p, None) == 0     # empty input: no launch


def test_workspace_sizes(q):
    # 2 MiB of back-pointers per tile at k = 2, V = 1, monotone in tiles
    w1, w2 = q.qtip_quantize_gpu_workspace(2, 1, 1), q.qtip_quantize_gpu_workspace(2, 1, 2)
    assert 2 << 20 <= w1 <= (2 << 20) + 4096 and w1 < w2 <= 2 * w1
    assert q.qtip_quantize_gpu_workspace(4, 2, 1) < w1
    assert q.qtip_quantize_gpu_workspace(1, 1, 1) == 0 and q.qtip_quantize_gpu_workspace(2, 1, 0) == 0


def test_binding_raises_with_message(q):
    with pytest.raises(q.QtipError) as e:
        q.qtip_decode_matvec(None, 16, 2, 1, 1, None, 16, 16, 0, 0, stream=0)
    assert e.value.code == -1 and "codes is NULL" in str(e.value)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2406_11235_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2406_11235_amd" not in text and "libqtip.so" not in text, f


C_PROGRAM = r"""
#include "qtip.h"
#include <stdio.h>
#include <string.h>
int main(void) {
    unsigned int word[16] = {0};
    float y[16];
    if (qtip_version() != QTIP_VERSION) return 1;
    /* n = 24 is not a multiple of 16: refused before any GPU work */
    if (qtip_decode_matvec(word, 16, 2, 1, QTIP_CODE_3INST, NULL, 16, 24, word, y, NULL) != QTIP_EINVAL) return 2;
    if (strlen(qtip_last_error()) == 0) return 3;
    if (qtip_quantize_gpu_workspace(2, 1, 1) == 0) return 4;
    puts("ok");
    return 0;
}
"""


def test_header_is_plain_c_and_the_library_links_from_c(q, tmp_path):
    """The boundary is usable without Python or C++: the header compiles as strict C99 (and as
    C++), and a C program linked against libqtip.so runs its argument checks on a machine
    without a GPU."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(q.library_path())
    src = tmp_path / "abi.c"
    src.write_text(C_PROGRAM)
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                   check=True)
    subprocess.run([shutil.which("g++") or "g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                    "-x", "c++", "-I", inc, str(src)], check=True)
    exe = tmp_path / "abi"
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lqtip",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert out.stdout.strip() == "ok"
