"""CPU-side checks: the C-ABI library loads, exports every declared symbol, and its
host-side argument checks answer without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2409_13761_amd import build, kdn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    build.ensure_built()
    return kdn.lib()


def test_a_library_built_from_other_sources_is_recognised(lib, tmp_path):
    """The binary carries the fingerprint of its sources; a changed comment in a copy of
    one source already makes the pair (binary, sources) stale."""
    want = build.source_fingerprint()
    assert build.library_fingerprint() == want and not build.is_stale()
    assert kdn.kdn_version().endswith("src:" + want)
    copies = []
    for f in build.SOURCES + build.HEADERS:
        c = tmp_path / os.path.basename(f)
        c.write_bytes(open(f, "rb").read())
        copies.append(str(c))
    assert build.source_fingerprint(copies) == want and not build.is_stale(files=copies)
    with open(copies[-2], "a") as fh:                      # one of the headers under csrc/
        fh.write("// a comment\n")
    assert build.source_fingerprint(copies) != want
    assert build.is_stale(files=copies)
    # a file that is no library of ours, or no file at all, counts as stale too
    other = tmp_path / "libother.so"
    other.write_bytes(b"\x7fELF no fingerprint here")
    assert build.library_fingerprint(str(other)) is None and build.is_stale(str(other))
    assert build.is_stale(str(tmp_path / "missing.so"))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(kdn_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(kdn.EXPORTS) == names


def test_chunk_bytes(lib):
    assert kdn.kdn_chunk_bytes(32, 8, 128, 1, 1) == 67584
    assert kdn.kdn_chunk_bytes(32, 8, 128, 1, 0) == 131072
    assert kdn.kdn_chunk_bytes(80, 8, 128, 1, 1) == 168960
    assert kdn.kdn_chunk_bytes(2, 4, 64, 256, 1) == 256 * 1088
    assert kdn.kdn_chunk_bytes(2, 4, 64, 0, 1) == 0
    assert kdn.kdn_chunk_bytes(2, 4, 64, 4, 7) == 0
    assert kdn.kdn_chunk_bytes(32, 8, 128, 1, 2) == 40960        # int4: 5 bits per element
    assert kdn.kdn_chunk_bytes(2, 4, 48, 4, 2) == 0              # int4 needs head_dim % 32 == 0
    assert kdn.kdn_chunk_bytes(32, 8, 128, 1, 3) == 67584        # fp8: the int8 footprint
    # 32768 tokens of the 80-layer shape need more than 32 bits
    assert kdn.kdn_chunk_bytes(80, 8, 128, 32768, 1) == 32768 * 168960


def _cache(**kw):
    d = dict(k=0x1000, v=0x2000, L=2, H=4, D=64, bs=16, nb=8)
    d.update(kw)
    H, D, bs, nb = d["H"], d["D"], d["bs"], d["nb"]
    return kdn.CacheDesc(d["k"], d["v"], d["L"], H, D, bs, nb,
                         d.get("ls", nb * bs * H * D), d.get("bst", bs * H * D),
                         d.get("ts", H * D), d.get("hs", D))


def _chunk(fmt=1, data=0x4000, T=16, L=2, H=4, D=64, nbytes=None):
    if nbytes is None:
        nbytes = kdn.kdn_chunk_bytes(L, H, D, T, fmt)
    return kdn.ChunkDesc(data, nbytes, fmt, L, H, D, T, 0, T)


def test_argument_errors_are_reported_on_the_host(lib):
    bt = 0x8000
    good = _cache()
    ch = _chunk()
    f = lib.kdn_store_chunk
    assert f(None, bt, 4, 0, 16, C.byref(ch), None) == kdn.EINVAL
    assert f(C.byref(good), None, 4, 0, 16, C.byref(ch), None) == kdn.EINVAL
    assert f(C.byref(good), bt, 4, 0, 0, C.byref(ch), None) == kdn.EINVAL          # empty range
    assert f(C.byref(good), bt, 4, -1, 16, C.byref(ch), None) == kdn.EINVAL
    assert f(C.byref(good), bt, 4, 60, 16, C.byref(ch), None) == kdn.ERANGE        # past the table
    assert f(C.byref(_cache(k=0x1008)), bt, 4, 0, 16, C.byref(ch), None) == kdn.EALIGN
    assert f(C.byref(_cache(hs=68)), bt, 4, 0, 16, C.byref(ch), None) == kdn.EALIGN
    assert f(C.byref(_cache(D=24)), bt, 4, 0, 16, C.byref(ch), None) == kdn.EUNSUPPORTED
    assert f(C.byref(_cache(D=1024)), bt, 4, 0, 16, C.byref(ch), None) == kdn.EUNSUPPORTED
    assert f(C.byref(good), bt, 4, 0, 16, C.byref(_chunk(nbytes=100)), None) == kdn.ESIZE
    assert f(C.byref(good), bt, 4, 0, 16, C.byref(_chunk(fmt=5, nbytes=1 << 20)), None) == kdn.EINVAL
    assert f(C.byref(good), bt, 4, 0, 16, C.byref(_chunk(data=0x4004)), None) == kdn.EALIGN
    assert f(C.byref(_cache(D=48)), bt, 4, 0, 16, C.byref(_chunk(fmt=2, D=48, nbytes=1 << 20)), None) == kdn.EUNSUPPORTED

    g = lib.kdn_load_chunk
    assert g(None, C.byref(good), bt, 4, 0, None) == kdn.EINVAL
    assert g(C.byref(ch), C.byref(good), bt, 4, 49, None) == kdn.ERANGE
    assert g(C.byref(_chunk(H=8)), C.byref(good), bt, 4, 0, None) == kdn.EINVAL   # shape mismatch
    short = _chunk()
    short.bytes -= 1
    assert g(C.byref(short), C.byref(good), bt, 4, 0, None) == kdn.ESIZE
    view = _chunk()
    view.token_start, view.num_tokens = 10, 10
    assert g(C.byref(view), C.byref(good), bt, 4, 0, None) == kdn.ERANGE

    off = (C.c_int32 * 2)(0, 16)
    arr = (kdn.ChunkDesc * 2)(_chunk(T=40), _chunk(T=40))
    h = lib.kdn_compose
    assert h(arr, off, 2, C.byref(good), bt, 4, 0, 10000.0, None) == kdn.ERANGE   # 80 tokens > 64 slots
    assert h(arr, off, 0, C.byref(good), bt, 4, 0, 10000.0, None) == kdn.EINVAL
    assert h(arr, None, 2, C.byref(good), bt, 4, 0, 10000.0, None) == kdn.EINVAL


def test_chunk_init_and_slice(lib):
    d = kdn.ChunkDesc()
    assert lib.kdn_chunk_init(C.byref(d), 0x4000, 1 << 20, 1, 2, 4, 64, 100) == kdn.OK
    assert (d.parent_tokens, d.token_start, d.num_tokens) == (100, 0, 100)
    s = kdn.ChunkDesc()
    assert lib.kdn_chunk_slice(C.byref(d), 10, 50, C.byref(s)) == kdn.OK
    s2 = kdn.ChunkDesc()
    assert lib.kdn_chunk_slice(C.byref(s), 5, 45, C.byref(s2)) == kdn.OK
    assert (s2.parent_tokens, s2.token_start, s2.num_tokens) == (100, 15, 45)
    assert lib.kdn_chunk_slice(C.byref(s), 5, 46, C.byref(s2)) == kdn.ERANGE
    assert lib.kdn_chunk_init(C.byref(d), 0x4000, 10, 1, 2, 4, 64, 100) == kdn.ESIZE
    assert lib.kdn_chunk_init(C.byref(d), 0x4001, 1 << 20, 1, 2, 4, 64, 100) == kdn.EALIGN


def test_status_strings(lib):
    for s in (0, -1, -2, -3, -4, -5, -6, -7):
        assert kdn.status_str(s)
    assert "kdn" in kdn.kdn_version()


def test_headers_are_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """The boundary is a C ABI: a C99 program that includes both headers compiles without a
    warning, links against the library and calls it (host-only entry points)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    src = tmp_path / "abi.c"
    src.write_text('#include "kdn.h"\n#include "kdn_pool.h"\n#include "kdn_arena.h"\n#include <stdio.h>\n'
                   'int main(void) {\n'
                   '    kdn_chunk c; char buf[16] __attribute__((aligned(16)));\n'
                   '    unsigned long long n = kdn_chunk_bytes(32, 8, 128, 1, KDN_FMT_INT8_ROWSCALE);\n'
                   '    int st = kdn_chunk_init(&c, buf, sizeof buf, KDN_FMT_RAW_BF16, 1, 1, 16, 1);\n'
                   '    kdn_arena_info ai; int a = kdn_arena_query(&ai);   /* no arena: not found, or no device */\n'
                   '    printf("%llu %d %d %u %s\\n", n, st, a, (unsigned)sizeof ai, kdn_status_str(KDN_ESIZE));\n'
                   '    return 0;\n}\n')
    exe = str(tmp_path / "abi")
    libdir = os.path.dirname(build.LIB_PATH)
    p = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", exe, "-L", libdir, "-lkdn", "-Wl,-rpath," + libdir],
                       capture_output=True, text=True)
    assert p.returncode == 0, p.stderr
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr
    got = out.stdout.split()
    assert got[:2] == ["67584", str(kdn.ESIZE)]
    assert int(got[2]) in (kdn.ENOTFOUND, kdn.EDEVICE)
    assert int(got[3]) == C.sizeof(kdn.ArenaInfo)          # the binding's struct is the header's


def test_arena_calls_check_their_arguments_before_any_device_work(lib):
    info = kdn.ArenaInfo()
    assert lib.kdn_arena_create(0, 0, C.byref(info)) == kdn.EINVAL           # no bytes
    assert lib.kdn_arena_create(1 << 30, 3, C.byref(info)) == kdn.EINVAL     # granule not a power of two
    assert lib.kdn_arena_create(1 << 30, 1024, C.byref(info)) == kdn.EINVAL  # granule above 512 MiB
    p = C.c_void_p()
    assert lib.kdn_arena_alloc(0, C.byref(p)) == kdn.EINVAL
    assert lib.kdn_arena_alloc(4096, None) == kdn.EINVAL
    assert lib.kdn_arena_free(None) == kdn.EINVAL
    assert lib.kdn_arena_query(None) == kdn.EINVAL
    # with no arena (or no device at all) nothing is handed out
    assert lib.kdn_arena_alloc(4096, C.byref(p)) in (kdn.ENOTFOUND, kdn.EDEVICE) and not p.value
    assert lib.kdn_arena_destroy() in (kdn.ENOTFOUND, kdn.EDEVICE)
