"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_path_does_not_import_the_oracle():
    """The package and bench.py's timed path never pull in oracle/ (only bench's cpu_baseline leg and
    the tests do): importing the package must not import it, and the package has no fallback."""
    code = "import sys; import paper_2101_05600_amd as m; print(any(k == 'oracle' or k.startswith('oracle.') for k in sys.modules))"
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120, cwd=ROOT)
    assert r.returncode == 0 and r.stdout.strip() == "False"
    src = open(os.path.join(ROOT, "paper_2101_05600_amd", "__init__.py")).read()
    assert "import oracle" not in src and "from oracle" not in src


def test_committed_counter_summaries_are_readable_by_the_bench_line():
    """The roofline object's profiler-side figures come from the committed summaries under profiles/:
    each must parse and carry traffic, the kernel's own duration and when it was measured."""
    sys.path.insert(0, ROOT)
    import bench
    for wl in ("cfg2", "cfg4b"):
        traffic, us, when = bench.read_profile_summary(os.path.join(ROOT, "profiles", f"k_score_{wl}_traffic.txt"))
        assert traffic and traffic > 1e6 and us and 1.0 < us < 1000.0 and when and "MI355X" in when
    assert bench.read_profile_summary(os.path.join(ROOT, "profiles", "no_such_file.txt")) == (None, None, None)
