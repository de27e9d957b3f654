"""Host-side checks of the benchmark's command line and of the build entry point (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         cwd=ROOT, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)
    assert not res.stdout.strip().startswith("{")              # no result line


def test_entry_points_exist_and_the_oracle_stays_out_of_the_product():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    assert callable(entry.build) and callable(entry.smoke)
    # nothing in the package imports the oracle or the scratch folder
    pkg = os.path.join(ROOT, "paper_2503_01586_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert "oracle" not in text.replace("no CPU fallback", ""), name
            assert "_work/" not in text and "_work\"" not in text, name
    # bench.py reaches the oracle only inside its cpu_baseline leg
    bench = open(os.path.join(ROOT, "bench.py")).read()
    head, _, tail = bench.partition("def cpu_baseline(")
    assert "from oracle" not in head and "import oracle" not in head
    assert "oracle" in tail
