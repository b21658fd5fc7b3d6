"""The C ABI without a GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any device work."""
import ctypes
import os
import re

import pytest

import paper_1803_11389_amd as ss

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ss.LIB_PATH):
        from paper_1803_11389_amd.build import build
        build()
    return ss.load_library()


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"}


def test_every_declared_symbol_is_exported(lib):
    """The method's interface (ssrnn.h) and the measurement aids (ssrnn_probe.h) are separate headers; the
    product header holds no process-wide setting."""
    for header, table in (("ssrnn.h", ss.EXPORTS), ("ssrnn_probe.h", ss.PROBE_EXPORTS)):
        names = _declared_symbols(header)
        assert names == set(table), header
        for n in names:
            assert getattr(lib, n) is not None
    assert "tune" not in open(os.path.join(ROOT, "include", "ssrnn.h")).read()


def test_version_and_workspace_query(lib):
    assert lib.ssrnn_version() >= 100
    assert ss.workspace_bytes(1, 128, 1, 4, ss.F32) >= 256
    one = ss.workspace_bytes(2, 1024, 2, 16, ss.F32)
    assert one >= 256 + (16 + 1) * 1024 * 4
    assert ss.workspace_bytes(0, 128, 1, 4, ss.F32) == 0
    assert ss.workspace_bytes(1, 128, 1, 0, ss.F32) == 0
    assert ss.workspace_bytes(1, 128, 1, 4, 7) == 0


def test_bad_arguments_fail_on_the_host(lib):
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below fails validation first
    tab = (ctypes.c_void_p * 1)(0x1000)
    args = dict(W=tab, bias=None, x=fake, c_init=None, h=fake, c_final=fake, n_layers=1, d=128, L=8, T=4,
                wdt=0, flags=0, ws=fake, ws_bytes=1 << 20, stream=None)

    def call(**kw):
        a = dict(args, **kw)
        return lib.sru_forward(a["W"], a["bias"], a["x"], a["c_init"], a["h"], a["c_final"], a["n_layers"],
                               a["d"], a["L"], a["T"], a["wdt"], a["flags"], a["ws"], a["ws_bytes"], a["stream"])

    assert call(W=None) == 1 and b"W is NULL" in lib.ssrnn_last_error()
    assert call(c_final=None) == 1
    assert call(x=None) == 1
    assert call(h=None) == 1
    assert call(n_layers=0) == 1
    assert call(d=0) == 1
    assert call(L=-1) == 1
    assert call(T=0) == 1
    assert call(wdt=5) == 1
    assert call(flags=1 << 20) == 1
    assert call(W=(ctypes.c_void_p * 1)(None)) == 1
    assert call(ws=None) == 3
    assert call(ws=ctypes.c_void_p(0x1010)) == 3                 # misaligned
    assert call(n_layers=2, W=(ctypes.c_void_p * 2)(0x1000, 0x1000), ws_bytes=512) == 3 and b"needed" in lib.ssrnn_last_error()
    q = lib.qrnn_forward(tab, None, fake, None, None, fake, fake, None, 1, 128, 8, 4, 0, 0, 0, fake, 1 << 20, None)
    assert q == 1                                               # k = 0
    assert call(flags=(1 << 8) | (2 << 4)) == 1 and b"packed" in lib.ssrnn_last_error()   # packed weights + vector-ALU kernel
    assert call(flags=1 << 8, d=100) == 2                        # no packed form for this width
    assert lib.ssrnn_linear_forward(None, fake, fake, 4, 4, 4, None) == 1
    assert lib.ssrnn_pack_weights(None, fake, 128, 1, 0, None) == 1
    assert lib.ssrnn_pack_weights(fake, fake, 128, 1, 0, None) == 1          # in place
    assert lib.ssrnn_pack_weights(fake, ctypes.c_void_p(0x2008), 128, 1, 0, None) == 1   # misaligned
    assert lib.ssrnn_pack_weights(fake, ctypes.c_void_p(0x2000), 100, 1, 0, None) == 2
    assert ss.packed_weight_bytes(128, 2, ss.F32) == 3 * 128 * 256 * 4
    assert ss.packed_weight_bytes(1024, 1, ss.BF16) == 3 * 1024 * 1024 * 2
    assert ss.packed_weight_bytes(100, 1, ss.F32) == 0 and ss.packed_weight_bytes(32, 1, ss.BF16) == 0
    # 8-bit weights: codes, padding to 256 bytes, one fp32 scale per row
    assert ss.weight_bytes(128, 1, ss.FP8) == 3 * 128 * 128 + 12 * 128
    assert ss.weight_bytes(10, 1, ss.FP8) == 512 + 120                      # 300 codes are padded to 512
    assert ss.weight_bytes(128, 2, ss.F32) == 3 * 128 * 256 * 4 and ss.weight_bytes(64, 1, ss.BF16) == 3 * 64 * 64 * 2
    assert ss.weight_bytes(0, 1, ss.FP8) == 0 and ss.weight_bytes(16, 1, 9) == 0
    assert ss.packed_weight_bytes(256, 1, ss.FP8) == ss.weight_bytes(256, 1, ss.FP8)
    assert ss.packed_weight_bytes(64, 1, ss.FP8) == 0                        # rows shorter than a 128-byte k-step
    assert ss.workspace_bytes(2, 1024, 2, 64, ss.FP8) == ss.workspace_bytes(2, 1024, 2, 64, ss.BF16)
    assert call(wdt=2, flags=3 << 4) == 2                                    # row-major 8-bit weights + matrix-core kernel
    assert call(flags=2) == 1                                                # no such schedule
    assert lib.ssrnn_read_probe(None, 1, 1024, 0, fake, None) == 1
    assert lib.ssrnn_read_probe(tab, 1, 1000, 0, fake, None) == 1            # not a multiple of 16 bytes
    assert lib.ssrnn_read_probe((ctypes.c_void_p * 1)(0x1004), 1, 1024, 0, fake, None) == 1
    assert lib.ssrnn_read_probe(tab, 9, 1024, 0, fake, None) == 1            # more buffers than a launch holds
    assert lib.ssrnn_read_probe(tab, 1, 1024, 0, None, None) == 1


def test_lstm_bad_arguments_fail_on_the_host(lib):
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below fails validation first
    tab = (ctypes.c_void_p * 1)(0x1000)
    args = dict(W=tab, U=tab, bias=None, x=fake, h_init=None, c_init=None, h=fake, h_final=fake, c_final=fake,
                n_layers=1, d=128, L=8, T=4, flags=0, ws=fake, ws_bytes=1 << 20, stream=None)

    def call(**kw):
        a = dict(args, **kw)
        return lib.lstm_forward(a["W"], a["U"], a["bias"], a["x"], a["h_init"], a["c_init"], a["h"], a["h_final"],
                                a["c_final"], a["n_layers"], a["d"], a["L"], a["T"], a["flags"], a["ws"], a["ws_bytes"],
                                a["stream"])

    assert call(W=None) == 1 and b"NULL" in lib.ssrnn_last_error()
    assert call(U=None) == 1
    assert call(U=(ctypes.c_void_p * 1)(None)) == 1
    assert call(h_final=None) == 1 and call(c_final=None) == 1
    assert call(x=None) == 1 and call(h=None) == 1
    assert call(n_layers=0) == 1 and call(d=0) == 1 and call(L=-1) == 1 and call(T=0) == 1
    assert call(flags=1) == 1
    assert call(d=1 << 17) == 2
    assert call(ws=None) == 1
    assert call(ws=ctypes.c_void_p(0x1010)) == 1                 # misaligned
    assert call(ws_bytes=512) == 3 and b"needed" in lib.ssrnn_last_error()
    need = lib.lstm_workspace_bytes(2, 1024, 64)
    # two copies of the layers' h, the input products of 16 steps, two hand-off blocks of 16 steps
    assert need >= 2 * 2 * 1024 * 4 + 16 * 4 * 1024 * 4 + 2 * 16 * 1024 * 4
    assert lib.lstm_workspace_bytes(2, 1024, 64) == lib.lstm_workspace_bytes(2, 1024, 16)
    assert lib.lstm_workspace_bytes(0, 1024, 4) == 0 and lib.lstm_workspace_bytes(1, 0, 4) == 0 and lib.lstm_workspace_bytes(1, 8, 0) == 0


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(ss, "_lib", None)
    monkeypatch.setattr(ss, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libssrnn.so"))
    with pytest.raises(ImportError):
        ss.load_library()
