"""Host-side parts of the benchmark contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_profiles_hold_text_summaries_with_their_commands():
    pdir = os.path.join(ROOT, "profiles")
    names = sorted(os.listdir(pdir))
    assert names, "profiles/ is empty"
    for n in names:
        assert n.endswith((".txt", ".md", ".json")), n
        assert os.path.getsize(os.path.join(pdir, n)) < 64 * 1024, n
        if n.endswith(".txt"):
            text = open(os.path.join(pdir, n)).read()
            assert "bench.py" in text, n          # the committed command that made it
