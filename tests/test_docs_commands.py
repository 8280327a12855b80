"""The commands quoted in profiles/ and the README must exist: every `bench.py --flag` they name is a
flag bench.py accepts, and every file they run is committed."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _documents():
    docs = [os.path.join(ROOT, "README.md"), os.path.join(ROOT, "DESIGN.md")]
    prof = os.path.join(ROOT, "profiles")
    docs += [os.path.join(prof, f) for f in sorted(os.listdir(prof)) if f.endswith((".md", ".txt"))]
    return docs


def test_bench_flags_named_in_the_documents_exist():
    help_text = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True,
                               check=True).stdout
    accepted = set(re.findall(r"--[a-z][a-z-]*", help_text))
    named = set()
    for path in _documents():
        for line in open(path):
            for m in re.finditer(r"bench\.py((?:\s+(?:--[a-z][a-z-]*|[A-Za-z0-9_|\[\].]+))+)", line):
                named |= set(re.findall(r"--[a-z][a-z-]*", m.group(1)))
    assert named, "no bench.py command found in the documents"
    assert named <= accepted, sorted(named - accepted)


def test_profiles_hold_text_summaries_only():
    prof = os.path.join(ROOT, "profiles")
    for f in os.listdir(prof):
        assert f.endswith((".md", ".txt")), f
        assert os.path.getsize(os.path.join(prof, f)) < 64 * 1024, f
        assert not re.search(r"round|r\d\d", f), f
