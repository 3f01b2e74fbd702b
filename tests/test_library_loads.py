"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header declares,
and its host-only entry points behave (no GPU work is issued here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "osscar.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(osscar_[a-z_]+)\s*\(", txt)))


def _lib():
    import paper_2403_12983_amd as pkg
    if not os.path.exists(pkg.lib_path()):
        from paper_2403_12983_amd import build
        build.build()
    return pkg, pkg.load_library()


def test_header_symbols_are_exported():
    pkg, lib = _lib()
    names = _declared()
    assert {"osscar_gram", "osscar_init_support", "osscar_local_search", "osscar_backsolve"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pkg.EXPORTED_SYMBOLS) == names


def test_binding_constants_equal_the_header_enums():
    """Every OSSCAR_* constant that the Python binding defines has the value the header gives it."""
    from paper_2403_12983_amd import binding as b
    txt = open(os.path.join(ROOT, "include", "osscar.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    header = {}
    for body in re.findall(r"enum\s*\{(.*?)\}", txt, flags=re.S):
        for name, val in re.findall(r"(OSSCAR_[A-Z0-9_]+)\s*=\s*(\d+)u?", body):
            header[name] = int(val)
    assert {"OSSCAR_SEARCH_ALWAYS_ACCEPT", "OSSCAR_SEARCH_EAGER", "OSSCAR_SEARCH_NO_LOOKAHEAD", "OSSCAR_SEARCH_EXACT_IN",
            "OSSCAR_F32", "OSSCAR_BF16"} <= set(header)
    mine = {n: getattr(b, n) for n in dir(b) if n.startswith("OSSCAR_") and isinstance(getattr(b, n), int)}
    assert mine, "the binding defines no constants?"
    for n, v in mine.items():
        assert n in header, n
        assert header[n] == v, (n, v, header[n])
    # the tensor ids the binding exposes as T_* (two of them under shorter names)
    alias = {"T_KEPT": "OSSCAR_T_KEPT_SLOTS", "T_CAND": "OSSCAR_T_CAND_SLOTS"}
    for n in dir(b):
        if n.startswith("T_") and isinstance(getattr(b, n), int):
            assert header[alias.get(n, "OSSCAR_" + n)] == getattr(b, n), n


def test_workspace_query_is_host_only_and_validates():
    pkg, lib = _lib()
    from paper_2403_12983_amd.binding import _Desc
    good = _Desc(28672, 7168, 28672, 1, 14336, 5000, 1, 1)
    nbytes = lib.osscar_workspace_bytes(C.byref(good))
    # H, G, N, Z in float32 are a lower bound
    assert nbytes > 4 * (2 * 28672 ** 2 + 2 * 28672 * 7168)
    assert nbytes < 40e9
    for bad in (_Desc(64, 32, 64, 2, 32, 10, 0, 0),      # d1 != p*q
                _Desc(64, 32, 64, 1, 65, 10, 0, 0),      # k > p
                _Desc(64, 32, 64, 1, 0, 10, 0, 0),       # k < 1
                _Desc(130, 32, 2, 65, 1, 10, 0, 0),      # q > 64
                _Desc(64, 32, 64, 1, 32, 10, 7, 0)):     # unknown dtype
        assert lib.osscar_workspace_bytes(C.byref(bad)) == 0
    ctx = C.c_void_p()
    assert lib.osscar_create(C.byref(ctx), C.byref(good), None, 0, None) == 1          # EINVAL: no workspace
    assert lib.osscar_create(C.byref(ctx), C.byref(good), C.c_void_p(256), 1024, None) == 2   # ENOMEM: too small
    assert lib.osscar_create(C.byref(ctx), C.byref(good), C.c_void_p(257), nbytes, None) == 1  # misaligned


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2403_12983_amd.binding as b
    monkeypatch.setattr(b, "_LIB", None)
    monkeypatch.setattr(b, "lib_path", lambda: str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        b.load_library()


@pytest.mark.parametrize("d1", [64, 328, 2048, 8192, 28672, 28700])
def test_gram_tile_schedule_covers_the_lower_triangle_once_and_balances_the_xcds(d1):
    import numpy as np
    pkg, lib = _lib()
    tiles = (d1 + 127) // 128
    n = lib.osscar_debug_tile_schedule(d1, None, 0)
    assert n > 0 and n % 8 == 0
    buf = (C.c_int32 * (2 * n))()
    assert lib.osscar_debug_tile_schedule(d1, buf, n) == n
    sched = np.frombuffer(buf, dtype=np.int32).reshape(n, 2)
    real = sched[sched[:, 0] >= 0]
    assert np.all(real[:, 1] <= real[:, 0]) and np.all(real >= 0) and np.all(real < tiles)
    assert len(real) == tiles * (tiles + 1) // 2
    assert len({(int(r), int(c)) for r, c in real}) == len(real)                      # every tile exactly once
    # the length the workspace query reserves for it
    assert n <= 8 * (tiles * tiles // 2 + tiles + 8)
    # workgroup i runs on XCD i % 8: equal work per XCD up to one strip of tile rows
    per_xcd = np.array([(sched[x::8, 0] >= 0).sum() for x in range(8)])
    assert per_xcd.max() - per_xcd.min() <= 4 * tiles
    if tiles >= 64:
        assert per_xcd.max() <= 1.05 * per_xcd.mean()
    # tiles that run together on an XCD (64 consecutive slots) share few column panels
    if tiles >= 64:
        x0 = sched[0::8][:64]
        x0 = x0[x0[:, 0] >= 0]
        assert len(set(x0[:, 0].tolist()) | set(x0[:, 1].tolist())) <= 24
    assert lib.osscar_debug_tile_schedule(0, None, 0) == -1
