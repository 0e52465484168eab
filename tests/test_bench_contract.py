"""Host-side checks of bench.py's command-line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, cwd=ROOT, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_bench_never_reaches_the_oracle_outside_the_cpu_baseline_leg():
    """The timed path must not import the oracle: its only use in bench.py is the cpu_baseline block."""
    src = open(os.path.join(ROOT, "bench.py")).read().splitlines()
    uses = [i for i, l in enumerate(src) if "oracle" in l and ("import" in l)]
    assert uses, "the cpu_baseline leg is expected to import the oracle"
    guard = [i for i, l in enumerate(src) if "no_cpu_baseline" in l and l.strip().startswith("if ")]
    assert guard and all(i > guard[0] for i in uses)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1909_03108_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            for line in open(os.path.join(pkg, name)):
                s = line.strip()
                assert not (s.startswith(("import oracle", "from oracle"))), (name, s)
