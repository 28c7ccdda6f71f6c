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
