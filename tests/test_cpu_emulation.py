"""The kernel SOURCES, run on the CPU under sanitizers (no GPU needed).

tests/cpu_emu builds the library's HIP files with g++ against a stand-in for the HIP runtime header:
work-groups run one after the other with one OS thread per work-item, barriers, 64-lane wave
operations (shuffles, ballots, DPP, readlane) and LDS emulated, "device memory" on the heap.  Small
batches are then decoded through the ordinary C ABI and compared with the oracle step by step, just
as the GPU tests do.  What this adds to them: AddressSanitizer and UBSan see every access the kernels
make (an index that leaves its array is an error here, not a fault on a shared machine),
ThreadSanitizer sees a missing barrier as a data race, and LDS starts out filled with a poison
pattern, so a kernel that reads what it has not written does not get zeros.  It says nothing about
speed and does not replace the GPU tests; "device memory" comes back from the allocator filled with
garbage, so a never-written value that steers an access is caught here (the real wave execution, memory model and intrinsics are
only there)."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
sys.path.insert(0, os.path.join(HERE, "cpu_emu"))

sys.path.insert(0, HERE)

import build_emu  # noqa: E402
from random_cases import CPU_SUBSET  # noqa: E402


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run(so, preload, env_extra, cases, timeout=900):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env.update(env_extra)
    env["OMP_NUM_THREADS"] = "1"
    r = subprocess.run([sys.executable, os.path.join(HERE, "cpu_emu", "run_case.py"), so, *cases],
                       capture_output=True, text=True, env=env, timeout=timeout)
    return r


def _preload_works(preload, env_extra):
    """Can a Python child start at all with this sanitizer runtime preloaded (it cannot in every
    environment: another preloaded library first, an unusual memory layout)?"""
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env.update(env_extra)
    try:
        r = subprocess.run([sys.executable, "-c", "import ctypes, numpy; print('probe ok')"],
                           capture_output=True, text=True, env=env, timeout=120)
    except subprocess.TimeoutExpired:
        return False
    return r.returncode == 0 and "probe ok" in r.stdout


ASAN_ENV = {"ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1:verify_asan_link_order=0",
            "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}
TSAN_ENV = {"TSAN_OPTIONS": "halt_on_error=0:report_signal_unsafe=0:history_size=2"}


PLANT = ("k_select.h",
         "  if (fs != 0 && fs < l) return;           // outputs of a finished utterance were settled when it finished\n"
         "  lds_barrier();",
         "  if (fs != 0 && fs < l) return;\n  /* planted mistake: no barrier here */")


@pytest.fixture(scope="module")
def runs(tmp_path_factory):
    """Builds the three instrumented libraries and runs their children, all side by side (a build takes
    most of a minute, a run about a minute, mostly waiting at emulated barriers).
    -> {name: CompletedProcess, or a string saying why it could not run}"""
    from concurrent.futures import ThreadPoolExecutor
    root = str(tmp_path_factory.mktemp("cpu_emu"))
    asan, tsan = _runtime("libasan.so"), _runtime("libtsan.so")
    plan = {
        "asan": (asan, ASAN_ENV, dict(sanitize=True),
                 ["windowed", "batch_window", "all_candidates", "all_candidates_few_ids", "logits_odd_vocab",
                  "pivot", "pivot_k80", "static_step", "radix_wide_ties", "wide_window_eos_run", "k80_eos_run"]),
        # the first steps of a fixed subset of the random configurations that tests/test_gpu_random_configs.py
        # decodes on the GPU (same table, tests/random_cases.py), device memory starting out as garbage
        "asan_random": (asan, ASAN_ENV, dict(sanitize=True), [f"random:{a}:{b}:{c}" for a, b, c in CPU_SUBSET]),
        # executor: the job queue with two host threads on two handles
        "tsan": (tsan, TSAN_ENV, dict(sanitize="thread"), ["windowed", "batch_window", "executor"]),
        "tsan_planted": (tsan, TSAN_ENV, dict(sanitize="thread", plant=PLANT), ["windowed"]),
    }

    def one(name):
        runtime, env, build_kw, cases = plan[name]
        if runtime is None:
            return "no such sanitizer runtime in this toolchain"
        if not _preload_works(runtime, env):
            return "a Python child does not start with this sanitizer runtime preloaded here"
        so = build_emu.build(os.path.join(root, name), **build_kw)
        return _run(so, runtime, env, cases)
    with ThreadPoolExecutor(max_workers=4) as ex:
        futs = {k: ex.submit(one, k) for k in plan}
        return {k: f.result() for k, f in futs.items()}


def _result(runs, name):
    r = runs[name]
    if isinstance(r, str):
        pytest.skip(r)
    return r, r.stdout + r.stderr


def test_kernels_under_address_and_ub_sanitizers(runs):
    r, out = _result(runs, "asan")
    assert r.returncode == 0, out[-4000:]
    assert "ERROR: AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert out.count("emu ok") == 11, out[-2000:]


def test_random_configurations_first_steps_under_address_sanitizer(runs):
    """The CPU side of the randomised GPU test: the same seeded cases (a fixed subset, first steps), on the
    kernel sources built for the CPU, under AddressSanitizer + UBSan, device memory poisoned."""
    r, out = _result(runs, "asan_random")
    assert r.returncode == 0, out[-4000:]
    assert "ERROR: AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert out.count("emu ok") == len(CPU_SUBSET), out[-2000:]


def test_kernels_under_thread_sanitizer(runs):
    r, out = _result(runs, "tsan")
    assert r.returncode == 0, out[-4000:]
    assert "WARNING: ThreadSanitizer" not in out, out[-6000:]
    assert out.count("emu ok") == 3, out[-2000:]


def test_thread_sanitizer_run_notices_a_missing_barrier(runs):
    """Self-test of the method: with the barrier between building the list keys and ranking them
    taken out of the (copied) split select kernel, the same run reports data races."""
    r, out = _result(runs, "tsan_planted")
    assert "WARNING: ThreadSanitizer: data race" in out and "k_select_split" in out, out[-3000:]
