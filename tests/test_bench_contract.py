"""Host-only checks of bench.py's contract: one GPU only, and the flags the committed profiles name exist."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert proc.returncode != 0
    assert "one GPU" in (proc.stderr + proc.stdout)
    env = dict(os.environ, WORLD_SIZE="2")
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert proc.returncode != 0 and "one GPU" in (proc.stderr + proc.stdout)


def test_every_flag_in_a_committed_profile_command_is_a_flag_of_bench():
    """The summaries under profiles/ give the command that made them; it has to stay runnable."""
    help_text = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120).stdout
    known = set(re.findall(r"(--[a-z][a-z0-9-]*)", help_text))
    prof_dir = os.path.join(ROOT, "profiles")
    seen = 0
    for name in sorted(os.listdir(prof_dir)):
        for line in open(os.path.join(prof_dir, name)):
            if "bench.py" not in line or "rocprofv3" not in line:
                continue
            flags = re.findall(r"(--[a-z][a-z0-9-]*)", line.split("bench.py", 1)[1])
            seen += 1
            assert set(flags) <= known, (name, set(flags) - known)
    assert seen >= 5


def test_product_and_oracle_share_no_code():
    """The library's Python side never imports the oracle, the oracle never imports the library, and bench.py reaches the
    oracle only inside its CPU-baseline leg."""
    pkg = os.path.join(ROOT, "paper_2510_25590_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "oracle/" not in text and "regione_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"^\s*(from|import)\s+paper_2510_25590_amd\b", text, re.M), f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"^\s*(from|import)\s+oracle\b", bench, re.M)]
    start = bench.index("def cpu_baseline(")
    end = bench.index("\ndef ", start + 1)
    assert uses and all(start < u < end for u in uses)
