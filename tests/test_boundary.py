"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports
every symbol the header declares, sizes follow the one-byte-per-parameter rule, and
argument validation rejects bad calls before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "quasar.h")


@pytest.fixture(scope="module")
def qb():
    from paper_2603_01399_amd import binding
    return binding


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(quasar_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported(qb):
    names = _declared_functions()
    assert len(names) >= 14
    assert set(names) == set(qb.EXPORTS)
    for n in names:
        assert hasattr(qb.lib(), n), n


def test_status_strings_and_version(qb):
    assert qb.status_string(0) == "ok"
    for s in range(1, 7):
        assert qb.status_string(s) not in ("ok", "unknown status")
    assert qb.status_string(99) == "unknown status"
    assert qb.version() >= 100


def test_sizes(qb):
    # Eq. 12 / Eq. 11: one byte per parameter for int8, two for bf16, no padding
    assert qb.packed_bytes(4096, 4096) == 4096 * 4096
    assert qb.packed_bytes_bf16(4096, 4096) == 2 * 4096 * 4096
    assert qb.packed_bytes(151936, 4096) == 622329856
    assert qb.packed_bytes(100, 4096) == 0 and qb.packed_bytes(4096, 100) == 0
    assert qb.workspace_bytes(8, 151936, 4096) > 0
    assert qb.workspace_bytes(33, 151936, 4096) == 0
    assert qb.workspace_bytes(0, 16, 64) == 0


def test_path_override(qb):
    assert qb.get_path() in (qb.PATH_AUTO, qb.PATH_VALU, qb.PATH_MFMA)
    before = qb.get_path()
    qb.set_path(qb.PATH_MFMA)
    assert qb.get_path() == qb.PATH_MFMA
    with pytest.raises(qb.QuasarError):
        qb.set_path(7)
    qb.set_path(before)


def test_argument_validation_without_launch(qb):
    L = qb.lib()
    vp = ctypes.c_void_p
    a = vp(0x1000)          # aligned fake device pointers: never dereferenced on the host
    odd = vp(0x1004)
    ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_WS, ERR_DTYPE = 1, 2, 3, 4, 5
    lin = L.quasar_w8_linear
    assert lin(None, 8, 1024, 1024, a, a, 1024, a, 1024, None, 0, None) == ERR_NULL
    assert lin(a, 8, 1024, 1024, a, None, 1024, a, 1024, None, 0, None) == ERR_NULL
    assert lin(a, 0, 1024, 1024, a, a, 1024, a, 1024, None, 0, None) == ERR_SHAPE
    assert lin(a, 33, 1024, 1024, a, a, 1024, a, 1024, None, 0, None) == ERR_SHAPE
    assert lin(a, 8, 1000, 1000, a, a, 1024, a, 1024, None, 0, None) == ERR_SHAPE      # K % 64
    assert lin(a, 8, 1024, 1024, a, a, 1000, a, 1000, None, 0, None) == ERR_SHAPE      # N % 16
    assert lin(a, 8, 1024, 512, a, a, 1024, a, 1024, None, 0, None) == ERR_SHAPE       # ldx < K
    assert lin(a, 8, 1024, 1028, a, a, 1024, a, 1024, None, 0, None) == ERR_SHAPE      # ldx % 8
    assert lin(odd, 8, 1024, 1024, a, a, 1024, a, 1024, None, 0, None) == ERR_ALIGN
    ver = L.quasar_lmhead_verify
    assert ver(a, 8, 1024, 1024, a, a, 4096, a, 9, a, a, a, 1 << 21, None) == ERR_SHAPE   # n_draft > M
    assert ver(a, 8, 1024, 1024, a, a, 4096, None, 3, a, a, a, 1 << 21, None) == ERR_NULL
    assert ver(a, 8, 1024, 1024, a, a, 4096, a, 7, a, a, None, 0, None) == ERR_WS
    assert ver(a, 8, 1024, 1024, a, a, 4096, a, 7, a, a, a, 16, None) == ERR_WS
    qz = L.quasar_quantize_weights
    assert qz(a, 7, 1024, 1024, 1024, a, a, None) == ERR_DTYPE
    assert qz(a, 0, 1024, 1024, 512, a, a, None) == ERR_SHAPE
    assert L.quasar_read_stream(a, 1000, a, None) == ERR_SHAPE
    assert L.quasar_copy_stream(a, None, 1024, None) == ERR_NULL


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more exits with a message instead of running."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr and res.stdout.strip() == ""


def test_sizes_of_the_newer_formats(qb):
    lib = qb.lib()
    # 4-bit: half a byte per weight + one bf16 step size per row and group of 128
    assert lib.quasar_w4_packed_bytes(4096, 4096) == 4096 * 4096 // 2 + 2 * 4096 * 32
    assert lib.quasar_w4_packed_bytes(4096, 4096 + 64) == 0 and lib.quasar_w4_packed_bytes(24, 128) == 0
    # key/value cache: keys and values, blocks of 32 positions x 128 x bf16 per kv head
    assert lib.quasar_kv_cache_bytes(8, 4096) == 2 * 8 * 128 * 8192
    assert lib.quasar_kv_cache_bytes(8, 4097) == 2 * 8 * 129 * 8192 and lib.quasar_kv_cache_bytes(8, 0) == 0
    # attention workspace: positive for valid shapes, 0 otherwise
    assert lib.quasar_attention_workspace_bytes(8, 32, 8, 4104) > 0
    assert lib.quasar_attention_workspace_bytes(8, 30, 8, 4104) == 0 and lib.quasar_attention_workspace_bytes(8, 32, 8, 4) == 0
    assert lib.quasar_sample_workspace_bytes(8, 151936) >= 8 * 151936 * 4
