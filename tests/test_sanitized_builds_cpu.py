"""The host-side code under sanitizers, on the CPU: the planner, the kernel body as the host emulation runs
it, the resource cache, the datatype tree / handle table / canonicalizer and the C oracle are rebuilt with
TP_SANITIZE=address (AddressSanitizer + UndefinedBehaviorSanitizer) or TP_SANITIZE=thread (ThreadSanitizer)
and a selection of the CPU tests runs against those builds in a child process that has the sanitizer's
runtime preloaded.  Any report fails the child.  The same switch works by hand for the whole CPU suite
(README: "Sanitizer builds").  Nothing of this runs on a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run_under(kind, runtimes, options, selection):
    libs = [_runtime(r) for r in runtimes]
    if not all(libs):
        pytest.skip(f"no {runtimes} in this toolchain")
    env = dict(os.environ)
    env["TP_SANITIZE"] = kind
    env.update(options)
    # the sanitizer's runtime has to come first; whatever was preloaded already stays behind it
    env["LD_PRELOAD"] = ":".join(libs + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *selection],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "Sanitizer" not in r.stdout + r.stderr, tail


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    _run_under("address", ["libasan.so", "libubsan.so"],
               {"ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1:abort_on_error=1",
                "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"},
               ["tests/test_resource_cache_cpu.py", "tests/test_library_cpu.py", "tests/test_oracle_pins.py", "-k",
                "cache or buffer_map or tile_shapes or random_types or splitting or abut or batch_of_different or "
                "grid_limit or multiply_shift or word_width or handle_table or tiny_type_maps_c or c_twin or roundtrip or "
                "threaded or truncation"])


def test_threaded_host_code_under_thread_sanitizer(tmp_path):
    # as a program of its own (tests/host_emul/sanitized_main.cpp): an interpreter in the process is
    # more than this sanitizer's runtime takes when it is preloaded
    if not _runtime("libtsan.so"):
        pytest.skip("no libtsan.so in this toolchain")
    csrc = os.path.join(ROOT, "paper_2012_14363_amd", "csrc")
    emul = os.path.join(ROOT, "tests", "host_emul")
    exe = str(tmp_path / "sanitized_main")
    oracle_obj = str(tmp_path / "typemap_oracle.o")
    flags = ["-O1", "-g", "-fsanitize=thread", "-fno-omit-frame-pointer", "-pthread"]
    subprocess.check_call(["gcc", "-std=c11", *flags, "-c", os.path.join(ROOT, "oracle", "typemap_oracle.c"), "-o", oracle_obj])
    subprocess.check_call(["g++", "-std=c++20", *flags, "-Wno-unknown-pragmas", "-I", csrc,
                           os.path.join(emul, "sanitized_main.cpp"), os.path.join(emul, "types_emul.cpp"),
                           os.path.join(emul, "cache_emul.cpp"), os.path.join(csrc, "type_tree.cpp"),
                           os.path.join(csrc, "canon.cpp"), os.path.join(csrc, "resource_cache.cpp"), oracle_obj, "-o", exe])
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:exitcode=66")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "ThreadSanitizer" not in r.stdout + r.stderr, (r.stdout + r.stderr)[-4000:]
    assert "handle table and commit: 0 wrong" in r.stdout and "resource cache: 0 wrong" in r.stdout
    assert "threaded oracle copy: equal" in r.stdout
