"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the
text-keyed index of the library and the C oracle are built with g++ / gcc and driven
by small native programs whose buffers have exact sizes."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _run(cmd, **kw):
    p = subprocess.run(cmd, capture_output=True, text=True, timeout=300, **kw)
    assert p.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), p.stdout[-2000:], p.stderr[-4000:])
    return p.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_pool_index_under_sanitizers(tmp_path):
    exe = str(tmp_path / "pool_fuzz")
    _run(["g++", "-std=c++17"] + SAN + ["-I", os.path.join(ROOT, "include"),
          os.path.join(ROOT, "tests", "native", "pool_fuzz.cpp"),
          os.path.join(ROOT, "paper_2409_13761_amd", "csrc", "kdn_pool.cpp"), "-o", exe])
    assert "pool_fuzz ok" in _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_check")
    _run(["gcc", "-std=c11", "-ffp-contract=off"] + SAN +
         [os.path.join(ROOT, "tests", "native", "oracle_check.c"),
          os.path.join(ROOT, "oracle", "kdn_oracle.c"), "-lm", "-o", exe])
    assert "oracle_check ok" in _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_arena_block_list_under_sanitizers(tmp_path):
    """The striped arena's bookkeeping (first fit, joining of freed neighbours, refusal of
    addresses that are no live block) needs no GPU: 60 000 random steps against a page map."""
    exe = str(tmp_path / "blocklist_fuzz")
    _run(["g++", "-std=c++17"] + SAN + ["-I", os.path.join(ROOT, "paper_2409_13761_amd", "csrc"),
          os.path.join(ROOT, "tests", "native", "blocklist_fuzz.cpp"), "-o", exe])
    assert "blocklist_fuzz ok" in _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
