"""The library's host-side logic (page tables and allocator, replay of device-side commits, the streaming
kernel's work plan) built for the CPU with the address and undefined-behaviour sanitizers and driven by
tests/host_fuzz.cpp.  No GPU, no HIP: the two headers are plain C++.

The same harness must also notice planted mistakes: copies of the headers with one line changed have to
make it fail, otherwise its checks would not be worth much."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_14889_amd", "csrc")
INCLUDE = os.path.join(ROOT, "include")
HARNESS = os.path.join(ROOT, "tests", "host_fuzz.cpp")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]


def build(tmp, header_dir, name="host_fuzz"):
    exe = os.path.join(tmp, name)
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", *SAN, f"-I{header_dir}", f"-I{INCLUDE}", HARNESS, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-3000:]
    return exe


def run(exe, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe, *map(str, args)], capture_output=True, text=True, timeout=300, env=env)


@pytest.fixture(scope="module")
def fuzz_exe(tmp_path_factory):
    return build(str(tmp_path_factory.mktemp("host_fuzz")), CSRC)


@pytest.mark.parametrize("seed", [1, 2, 20260414])
def test_tables_and_plans_hold_under_sanitizers(fuzz_exe, seed):
    res = run(fuzz_exe, seed, 20000, 1500)
    assert res.returncode == 0, (res.stdout + res.stderr)[-3000:]
    assert "held" in res.stdout


MUTANTS = [
    # (header, the line as it is, the planted mistake)
    ("host_tables.h", "const int page = *free_pages.begin();\n        free_pages.erase(free_pages.begin());",
     "const int page = *free_pages.rbegin();\n        free_pages.erase(page);"),                       # highest free page instead of the lowest
    ("host_tables.h", "if (pending_pt[i] == seq && pending_pt[i + 1] == -1) {", "if (false) {"),             # two length entries in one batch
    ("host_tables.h", "for (size_t i = keep; i < pt[s].size(); ++i) free_pages.insert(pt[s][i]);", ""),     # cut pages leak
    ("host_tables.h", "if (seq < 0 || seq >= max_seqs || !live[seq] || !free_pages.count(page)) return false;",
     "if (seq < 0 || seq >= max_seqs || !free_pages.count(page)) return false;"),                           # log may name a dead sequence
    ("plan.h", "if (t1 > lens[b]) t1 = lens[b];", ""),                                                      # last segment past the end
    ("plan.h", "s.part += part_begin[s.b];", ""),                                                           # partial slots not rebased
    ("plan.h", "const int pg0 = (t0 >> 4) + 2 * tc;", "const int pg0 = (t0 >> 4) + tc;"),                   # wrong first page of a wave
    ("plan.h", "left -= take;\n                at += take;", "left -= take;\n                at += take + (it == 1);"),   # a tile skipped
]


@pytest.mark.parametrize("header,old,new", MUTANTS, ids=[f"{m[0]}-{i}" for i, m in enumerate(MUTANTS)])
def test_planted_mistakes_are_caught(tmp_path, header, old, new):
    hdr_dir = tmp_path / "csrc"
    hdr_dir.mkdir()
    for h in ("host_tables.h", "plan.h"):
        shutil.copy(os.path.join(CSRC, h), hdr_dir / h)
    text = (hdr_dir / header).read_text()
    assert text.count(old) == 1, f"the line to change is no longer in {header}"
    (hdr_dir / header).write_text(text.replace(old, new))
    exe = build(str(tmp_path), str(hdr_dir), "mutant")
    res = run(exe, 1, 8000, 600)
    assert res.returncode != 0, "the harness did not notice: " + old
