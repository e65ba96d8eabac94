"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; GPU code is never
instrumented): the C oracle runs its pins once as a sanitizer build, and the host side of
libtide_route -- argument checks, the prefill plan, the persistent kernels' tile schedule, the
workspace arithmetic -- runs the plan and boundary tests as a sanitizer build of the same sources."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_FLAGS = "-fsanitize=address,undefined -fno-sanitize-recover=undefined -fno-omit-frame-pointer -g -O1"


def _tool_file(tool, name):
    out = subprocess.run([tool, f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def _sanitizer_env(runtime, log_dir, **extra):
    """The sanitizer runtime must be the first library the interpreter loads; whatever is preloaded already stays.
    Reports go to files under log_dir (pytest captures the child's stderr and a report dies with the process)."""
    preload = runtime + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    log = os.path.join(str(log_dir), "sanitizer")
    return dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS=f"detect_leaks=0:verify_asan_link_order=0:log_path={log}",
                UBSAN_OPTIONS=f"halt_on_error=1:print_stacktrace=1:log_path={log}", PYTHONDONTWRITEBYTECODE="1", **extra)


def _reports(log_dir):
    return "".join(open(os.path.join(str(log_dir), f)).read() for f in sorted(os.listdir(str(log_dir))) if f.startswith("sanitizer"))


def _pytest(files, env, timeout):
    return subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", *files], cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=timeout)


def _clean(run, log_dir):
    text = run.stdout + run.stderr + _reports(log_dir)
    return run.returncode == 0 and "AddressSanitizer" not in text and "runtime error:" not in text


@pytest.fixture(scope="module")
def gcc_asan():
    lib = _tool_file("gcc", "libasan.so")
    if lib is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    return lib


def _oracle_copy(tmp_path, name):
    parent = tmp_path / name
    shutil.copytree(os.path.join(ROOT, "oracle"), parent / "oracle", ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    return parent


def test_oracle_pins_under_sanitizers(gcc_asan, tmp_path):
    parent = _oracle_copy(tmp_path, "san")
    env = _sanitizer_env(gcc_asan, tmp_path, TIDE_ORACLE_PARENT=str(parent), TIDE_ORACLE_CFLAGS=SAN_FLAGS)
    run = _pytest([os.path.join(ROOT, "tests", "test_oracle_pins.py")], env, 900)
    assert _clean(run, tmp_path), run.stdout[-3000:] + run.stderr[-3000:] + _reports(tmp_path)[-3000:]
    assert (parent / "oracle" / "libtide_oracle.so").exists()          # the instrumented copy is what ran


def test_sanitizer_build_catches_a_planted_overflow(gcc_asan, tmp_path):
    """Control: the same mechanism fails when the oracle copy allocates one element too few for a heap array."""
    parent = _oracle_copy(tmp_path, "ovf")
    src = parent / "oracle" / "tide_oracle.c"
    text = src.read_text()
    site = "double* act = (double*)malloc(sizeof(double) * (size_t)b);"
    assert site in text
    src.write_text(text.replace(site, "double* act = (double*)malloc(sizeof(double) * (size_t)(b - 1));"))
    env = _sanitizer_env(gcc_asan, tmp_path, TIDE_ORACLE_PARENT=str(parent), TIDE_ORACLE_CFLAGS=SAN_FLAGS)
    run = _pytest([os.path.join(ROOT, "tests", "test_oracle_pins.py")], env, 900)
    assert run.returncode != 0 and "heap-buffer-overflow" in _reports(tmp_path), run.stdout[-2000:] + _reports(tmp_path)[-2000:]


def test_host_side_of_the_library_under_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    runtime = _tool_file(hipcc, "libclang_rt.asan-x86_64.so") if os.path.exists(hipcc) else None
    if runtime is None:
        pytest.skip("hipcc or clang's AddressSanitizer runtime is not installed")
    from paper_2603_21365_amd.build import CSRC, HIPCC_FLAGS, INCLUDE
    lib = str(tmp_path / "libtide_route_hostsan.so")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"]
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        host_san += ["-Xarch_host", f]                               # host pass only: device code stays uninstrumented
    cmd = [hipcc, *flags, "-O1", "-g", *host_san, "-shared-libsan", "-I", INCLUDE, "-o", lib, os.path.join(CSRC, "tide_route.hip")]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert build.returncode == 0, build.stderr[-3000:]
    env = _sanitizer_env(runtime, tmp_path, TIDE_ROUTE_LIB=lib)
    run = _pytest([os.path.join(ROOT, "tests", "test_plan.py"), os.path.join(ROOT, "tests", "test_abi.py")], env, 900)
    assert _clean(run, tmp_path), run.stdout[-3000:] + run.stderr[-3000:] + _reports(tmp_path)[-3000:]
    assert " passed" in run.stdout
