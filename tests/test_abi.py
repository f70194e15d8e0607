"""Host-only checks of the C ABI: the library loads, exports what include/fnn.h declares,
and rejects bad arguments before touching the device (no GPU needed)."""
import ctypes
import os
import re
import shutil
import subprocess

import pytest

import paper_2503_10017_amd as fnn
from paper_2503_10017_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fnn.library_path()):
        from paper_2503_10017_amd import build
        build.build()
    return fnn.load_library()


def declared_functions(header="fnn.h"):
    with open(os.path.join(ROOT, "include", header)) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fnn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert names == ["fnn_blocked_workspace_bytes", "fnn_mutual_dense", "fnn_nearest", "fnn_nearest_blocked",
                     "fnn_pairs_to_pixels", "fnn_reciprocal", "fnn_reciprocal_static", "fnn_status_string",
                     "fnn_workspace_bytes", "fnn_workspace_bytes_opts"]
    measure = declared_functions("fnn_measure.h")
    assert measure == ["fnn_measure_ceiling", "fnn_trace_begin", "fnn_trace_end", "fnn_trace_kind_name"]
    for name in names + measure:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = {fnn.fnn_status_string(code) for code in range(8)}
    assert len(seen) == 8
    assert fnn.fnn_status_string(0) == "ok"
    assert fnn.fnn_status_string(99) == "unknown status"


def test_workspace_bytes(lib):
    small = fnn.fnn_workspace_bytes(1, 3072, 3072, 24, 48, "f16")
    big = fnn.fnn_workspace_bytes(1, 196608, 196608, 24, 3072, "f16")
    batch = fnn.fnn_workspace_bytes(16, 196608, 196608, 24, 3072, "f16")
    assert 0 < small < big < batch
    assert big >= 2 * 196608 * 24 * 2                      # two prepared 16-bit maps, 24 channels unpadded
    assert fnn.fnn_workspace_bytes(1, 196608, 196608, 24, 3072, "f32") > big
    assert fnn.fnn_workspace_bytes(0, 10, 10, 24, 1, "f16") == 0     # batch out of range
    assert fnn.fnn_workspace_bytes(1, 10, 10, 33, 1, "f16") == 0     # d out of range
    assert fnn.fnn_workspace_bytes(1, -1, 10, 24, 1, "f16") == 0
    assert fnn.fnn_workspace_bytes(65, 10, 10, 24, 1, "f16") == 0
    # the options-aware query: no flag = the plain one; squared distance widens 24-channel rows to 32
    assert fnn.fnn_workspace_bytes_opts(1, 196608, 196608, 24, 3072, "f16") == big
    assert fnn.fnn_workspace_bytes_opts(1, 196608, 196608, 24, 3072, "f16", l2=True) >= big + 2 * 196608 * 8 * 2
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 29, 8, "f16", l2=True) == 0      # 29 + 4 channels do not fit
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 12, 8, "f16", l2=True) == fnn.fnn_workspace_bytes_opts(1, 64, 64, 16, 8, "f16")
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 24, 8, "f16", max_iter=-1) == 0  # invalid options
    # two-term representation: 3 * 24 channels padded to 80 instead of 24; every d up to 32 fits; fp16 products only
    assert fnn.fnn_workspace_bytes_opts(1, 196608, 196608, 24, 3072, "f16", split=True) >= big + 2 * 196608 * (80 - 24) * 2
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 32, 8, "f16", split=True) > 0
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 24, 8, "bf16", split=True) == 0
    assert fnn.fnn_workspace_bytes_opts(1, 64, 64, 24, 8, "f16", split=True, l2=True) == 0


def _map(n=64, d=24, dtype=0, stride=None, data=0x1000):
    arr = (binding._Map * 1)()
    arr[0].data = data
    arr[0].n = n
    arr[0].d = d
    arr[0].dtype = dtype
    arr[0].row_stride = d if stride is None else stride
    return arr


def _opts(compute=1, max_iter=10, reserved0=0, flags=0):
    o = binding._Opts()
    o.compute = compute
    o.max_iter = max_iter
    o.flags = flags
    o.reserved[0] = reserved0
    return o


def _nearest(lib, src, tgt, opts, nq=8, out=0x2000, ws=0x10000, ws_bytes=1 << 30, q_idx=None, batch=1):
    vp = ctypes.c_void_p
    return lib.fnn_nearest(batch, ctypes.cast(src, vp) if src is not None else None, q_idx, nq, None,
                           ctypes.cast(tgt, vp) if tgt is not None else None,
                           ctypes.byref(opts) if opts is not None else None, vp(out) if out else None, None,
                           vp(ws) if ws else None, ws_bytes, None)


def test_argument_errors_are_caught_on_the_host(lib):
    # fake, never dereferenced device addresses: every call below must fail before any launch
    ok_map, opts = _map(), _opts()
    assert _nearest(lib, None, ok_map, opts) == 1                      # FNN_E_NULL
    assert _nearest(lib, ok_map, ok_map, None) == 1
    assert _nearest(lib, ok_map, ok_map, opts, out=0) == 1
    assert _nearest(lib, _map(data=0), ok_map, opts) == 1
    assert _nearest(lib, ok_map, ok_map, opts, batch=0) == 2           # FNN_E_SHAPE
    assert _nearest(lib, ok_map, ok_map, opts, batch=65) == 2
    assert _nearest(lib, _map(d=33), ok_map, opts) == 2
    assert _nearest(lib, _map(d=16), ok_map, opts) == 2                # d mismatch
    assert _nearest(lib, _map(stride=8), ok_map, opts) == 2            # row_stride < d
    assert _nearest(lib, ok_map, ok_map, opts, nq=65) == 2             # nq > n without q_idx
    assert _nearest(lib, ok_map, ok_map, opts, nq=-1) == 2
    assert _nearest(lib, _map(dtype=7), ok_map, opts) == 3             # FNN_E_DTYPE
    assert _nearest(lib, ok_map, ok_map, _opts(compute=5)) == 3
    assert _nearest(lib, ok_map, ok_map, _opts(max_iter=-1)) == 4      # FNN_E_RANGE
    assert _nearest(lib, ok_map, ok_map, _opts(reserved0=1)) == 4
    assert _nearest(lib, ok_map, ok_map, _opts(flags=16)) == 4         # unknown flag
    assert _nearest(lib, ok_map, ok_map, _opts(compute=2, flags=8)) == 7   # two-term representation: fp16 products only
    assert _nearest(lib, ok_map, ok_map, _opts(compute=0, flags=8)) == 7
    assert _nearest(lib, ok_map, ok_map, _opts(flags=12)) == 7         # ... and not with the squared distance
    assert _nearest(lib, ok_map, ok_map, _opts(flags=2)) == 7          # FNN_E_UNSUPPORTED: fp16 accumulation is blocked-only
    assert _nearest(lib, _map(d=29), _map(d=29), _opts(flags=4)) == 2  # squared distance: 29 + 4 channels do not fit
    assert _nearest(lib, _map(d=31), _map(d=31), _opts(compute=0, flags=4)) == 2
    assert _nearest(lib, ok_map, ok_map, _opts(flags=6)) == 7          # fp16 accumulation wins: unsupported here
    assert _nearest(lib, ok_map, ok_map, opts, ws=0) == 5              # FNN_E_WORKSPACE
    assert _nearest(lib, ok_map, ok_map, opts, ws=0x10001) == 5        # misaligned
    assert _nearest(lib, ok_map, ok_map, opts, ws_bytes=16) == 5       # too small
    assert _nearest(lib, ok_map, ok_map, opts, nq=0) == 0              # nothing to do is fine


def test_reciprocal_and_dense_argument_errors(lib):
    vp = ctypes.c_void_p
    m, o = _map(), _opts()
    cm = ctypes.cast(m, vp)

    def recip(d1=cm, d2=cm, seeds=vp(0x3000), n_seeds=4, opts=o, outs=0x4000, n_pairs=0x5000, ws=0x10000, wsb=1 << 30):
        return lib.fnn_reciprocal(1, d1, d2, seeds, n_seeds, ctypes.byref(opts) if opts is not None else None,
                                  vp(outs) if outs else None, vp(outs) if outs else None, vp(outs) if outs else None,
                                  vp(outs) if outs else None, vp(n_pairs) if n_pairs else None,
                                  vp(ws) if ws else None, wsb, None)

    assert recip(d1=None) == 1
    assert recip(seeds=None) == 1
    assert recip(outs=0) == 1
    assert recip(n_pairs=0) == 1
    assert recip(n_seeds=-3) == 2
    assert recip(d2=ctypes.cast(_map(d=8), vp)) == 2
    assert recip(d2=ctypes.cast(_map(n=0, data=0), vp)) == 2           # seeds but an empty image
    assert recip(opts=_opts(max_iter=-2)) == 4
    assert recip(wsb=128) == 5

    def dense(d1=cm, d2=cm, opts=o, outs=0x4000, n_pairs=0x5000, ws=0x10000, wsb=1 << 30):
        return lib.fnn_mutual_dense(1, d1, d2, ctypes.byref(opts) if opts is not None else None,
                                    vp(outs) if outs else None, None, vp(outs) if outs else None, None,
                                    vp(outs) if outs else None, vp(n_pairs) if n_pairs else None,
                                    vp(ws) if ws else None, wsb, None)

    assert dense(d1=None) == 1
    assert dense(outs=0) == 1
    assert dense(n_pairs=0) == 1
    assert dense(d2=ctypes.cast(_map(d=8), vp)) == 2
    big = ctypes.cast(_map(n=(1 << 30) + 1), vp)
    assert dense(d1=big, d2=big) == 2                                   # the dense mode stops at 2^30 pixels
    assert dense(opts=_opts(compute=-1)) == 3
    assert dense(ws=0) == 5


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope" / "libfnn.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()


def test_pairs_to_pixels_argument_errors(lib):
    vp, f = ctypes.c_void_p, ctypes.c_float

    def call(batch=1, pairs=0x1000, n_pairs=0x2000, max_pairs=16, n=64, w1=8, m=64, w2=8, out=0x3000, count=0x4000):
        return lib.fnn_pairs_to_pixels(batch, vp(pairs) if pairs else None, vp(n_pairs) if n_pairs else None, max_pairs,
                                       n, w1, m, w2, None, None, f(0.0), f(0.0), vp(out) if out else None,
                                       vp(count) if count else None, None)

    assert call(batch=0) == 2 and call(batch=65) == 2
    assert call(w1=0) == 2 and call(w2=-3) == 2 and call(max_pairs=-1) == 2 and call(n=-1) == 2
    assert call(n_pairs=0) == 1 and call(count=0) == 1 and call(pairs=0) == 1 and call(out=0) == 1


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_header_is_plain_c_and_usable_from_a_c_program(tmp_path):
    here = os.path.dirname(os.path.abspath(__file__))
    exe = str(tmp_path / "c_abi_check")
    build = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(here, "..", "include"),
                            os.path.join(here, "c_abi_check.c"), "-o", exe, "-ldl"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe, binding.load_library()._name], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "c abi ok" in run.stdout, run.stdout + run.stderr
