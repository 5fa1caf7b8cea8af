"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""          # no result line


def test_product_path_does_not_import_the_oracle():
    # only the cpu_baseline leg of bench.py may touch oracle/; the package itself never does
    pkg = os.path.join(ROOT, "paper_2602_23999_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            src = open(os.path.join(pkg, name)).read()
            assert "from oracle" not in src and "import oracle" not in src, name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    head, _, tail = bench.partition("def cpu_baseline(")
    body, _, rest = tail.partition("\ndef ")
    assert "from oracle" not in head and "import oracle" not in head
    assert "from oracle" not in rest and "import oracle" not in rest
    assert "from oracle" in body
