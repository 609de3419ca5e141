"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol include/spdnn.h declares, sizes arenas sensibly, and rejects bad
arguments with error codes (argument checks run before any HIP call)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2007_14152_amd as sp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "spdnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spdnn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sp.lib()
    names = declared_symbols()
    assert set(names) == set(sp.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_arena_sizes():
    w = sp.spdnn_weights_bytes(1024, 120)
    # at least u16 index + fp32 value per connection, plus the bias
    assert w >= 120 * 1024 * 32 * 6 + 1024 * 4
    assert w < 120 * 1024 * 32 * 6 * 1.2 + (1 << 20)
    k = sp.spdnn_work_bytes(1024, 1000)
    assert k >= 2 * 1000 * 1024 * 4 + 4 * 1000 * 4 + 2 * 1000   # two feature maps, four row lists, two byte flags per row
    assert sp.spdnn_work_bytes(65536, 60000) >= 2 * 60000 * 65536 * 4
    assert sp.spdnn_work_bytes(64, 0) > 0
    # windows of one LDS stage need no more than the compact layout; wider ones do
    n = 16384
    compact = sp.spdnn_weights_bytes_for_window(n, 10, 4096)
    assert compact == sp.spdnn_weights_bytes_for_window(n, 10, 1024)
    assert compact < sp.spdnn_weights_bytes_for_window(n, 10, 8192) <= sp.spdnn_weights_bytes_for_window(n, 10, 12288)
    assert sp.spdnn_weights_bytes_for_window(n, 10, 12288) <= sp.spdnn_weights_bytes_for_window(n, 10, n)
    assert sp.spdnn_weights_bytes_for_window(n, 10, n) == sp.spdnn_weights_bytes(n, 10)
    assert sp.spdnn_weights_bytes(65536, 2) < 2 * 65536 * 32 * 6 * 8


@pytest.mark.parametrize("N,L", [(0, 1), (16, 1), (34, 1), (65540, 1), (64, 0), (-4, 3)])
def test_bad_shapes_are_rejected(N, L):
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_weights_bytes(N, L)
    assert e.value.code == sp.SPDNN_EINVAL
    assert sp.spdnn_last_error() != ""


def test_null_and_negative_arguments():
    L = sp.lib()
    assert L.spdnn_weights_bytes(64, 1, None) == sp.SPDNN_EINVAL
    assert L.spdnn_work_bytes(64, -1, ctypes.byref(ctypes.c_size_t())) == sp.SPDNN_EINVAL
    assert L.spdnn_destroy(None) == sp.SPDNN_OK
    n = ctypes.c_int32(7)
    assert L.spdnn_infer(None, None, 0, None, 0, ctypes.byref(n), None, None) == sp.SPDNN_EINVAL
    assert L.spdnn_set_profiling(None, 1) == sp.SPDNN_EINVAL


def _host_model(N, L, bias_value=-0.1):
    idx = [np.tile(np.arange(32, dtype=np.int32), (N, 1)) for _ in range(L)]
    val = [np.full((N, 32), 0.0625, dtype=np.float32) for _ in range(L)]
    bias = np.full(N, bias_value, dtype=np.float32)
    return idx, val, bias


def test_create_rejects_before_touching_the_gpu():
    N, L = 64, 2
    idx, val, bias = _host_model(N, L)
    ip = [a.ctypes.data for a in idx]
    vp = [a.ctypes.data for a in val]
    need = sp.spdnn_weights_bytes(N, L)
    fake_arena = 256 * 4096          # an aligned, non-null address that is never dereferenced
    for kwargs, code in [
        (dict(arena_ptr=0), sp.SPDNN_EINVAL),
        (dict(arena_ptr=fake_arena + 8), sp.SPDNN_EINVAL),
        (dict(arena_bytes=need - 1), sp.SPDNN_ESIZE),
        (dict(where=5), sp.SPDNN_EINVAL),
        (dict(idx_ptrs=[ip[0], 0]), sp.SPDNN_EINVAL),
    ]:
        args = dict(N=N, L=L, idx_ptrs=ip, val_ptrs=vp, bias_ptr=bias.ctypes.data, where=sp.SPDNN_HOST,
                    arena_ptr=fake_arena, arena_bytes=need)
        args.update(kwargs)
        with pytest.raises(sp.SpdnnError) as e:
            sp.spdnn_create(**args)
        assert e.value.code == code, kwargs


def test_positive_bias_is_rejected():
    """Dropping all-zero rows is exact only if a zero row stays zero, i.e. bias <= 0."""
    N, L = 64, 1
    idx, val, bias = _host_model(N, L)
    bias[17] = 0.25
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_create(N, L, [a.ctypes.data for a in idx], [a.ctypes.data for a in val], bias.ctypes.data,
                        sp.SPDNN_HOST, 256 * 4096, sp.spdnn_weights_bytes(N, L))
    assert e.value.code == sp.SPDNN_EBIAS
    assert "bias[17]" in sp.spdnn_last_error()
    bias[17] = np.nan
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_create(N, L, [a.ctypes.data for a in idx], [a.ctypes.data for a in val], bias.ctypes.data,
                        sp.SPDNN_HOST, 256 * 4096, sp.spdnn_weights_bytes(N, L))
    assert e.value.code == sp.SPDNN_EBIAS


def test_header_is_plain_c_and_a_c_program_links():
    """include/spdnn.h compiles as C99 on its own, and the C user of the ABI builds and links
    against the library (it runs in the GPU tests)."""
    import subprocess
    import sys
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-x", "c",
                    os.path.join(ROOT, "include", "spdnn.h")], check=True)
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g
    exe = g.build_c_check()
    assert os.path.exists(exe)


def test_no_library_no_product_and_no_oracle_in_the_product():
    """Without csrc/libspdnn.so the binding raises (there is no CPU path to fall back to), and
    nothing under the package imports or names the oracle."""
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "import paper_2007_14152_amd as sp\n"
            "from paper_2007_14152_amd import build as b\n"
            "b.LIB = b.LIB + '.absent'\n"
            "try:\n"
            "    sp.spdnn_weights_bytes(64, 1)\n"
            "except RuntimeError as e:\n"
            "    assert 'no fallback' in str(e), e\n"
            "    assert 'oracle' not in sys.modules\n"
            "    print('raised')\n" % ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert out.returncode == 0 and "raised" in out.stdout, out.stdout + out.stderr
    pkg = os.path.join(ROOT, "paper_2007_14152_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "import oracle" not in text and "from oracle" not in text and "spdnn_oracle" not in text, f
