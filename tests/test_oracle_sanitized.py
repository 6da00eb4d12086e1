"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer: the pins of
tests/test_oracle_pins.py and the queue-size tests run once more, in a child process, against a
build of oracle/mqg_oracle.c with -fsanitize=address,undefined.  An out-of-bounds access, a use
after free, a signed overflow or a misaligned access anywhere the pins reach aborts the child."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_pins(lib, log_path, *selection):
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's libasan.so not found"
    env = dict(os.environ)
    # the sanitizer runtime has to be loaded before the interpreter's own libraries
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = f"detect_leaks=0:halt_on_error=1:log_path={log_path}"   # CPython itself leaks at exit
    env["UBSAN_OPTIONS"] = f"halt_on_error=1:print_stacktrace=1:log_path={log_path}"
    env["MQG_ORACLE_LIB"] = lib
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *selection]
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)


def reports(log_path):
    d, base = os.path.split(log_path)
    return "".join(open(os.path.join(d, f)).read() for f in sorted(os.listdir(d)) if f.startswith(base + "."))


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = oracle.build_sanitized(os.path.join(ROOT, "_build"))
    log_path = str(tmp_path / "san")
    proc = run_pins(lib, log_path, os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_queue_size.py"))
    tail = "\n".join(proc.stdout.splitlines()[-40:])
    assert proc.returncode == 0, tail
    assert " passed" in tail and reports(log_path) == "", reports(log_path)[:4000]


def test_a_planted_overflow_in_the_oracle_is_caught(tmp_path):
    """The check above can fail: a copy of the source that reads one element past an array (planted
    here, on the CPU, in the oracle) aborts the same run."""
    src = open(os.path.join(ROOT, "oracle", "mqg_oracle.c")).read()
    good = "for (int64_t i = 0; i < num_nodes; ++i) scores[i] = cur[i];"
    assert src.count(good) == 1
    bad_c = tmp_path / "planted.c"
    bad_c.write_text(src.replace(good, "for (int64_t i = 0; i <= num_nodes; ++i) scores[i] = cur[i];"))
    lib = str(tmp_path / "libplanted.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-o", lib, str(bad_c), "-lm"])
    log_path = str(tmp_path / "san")
    proc = run_pins(lib, log_path, os.path.join(ROOT, "tests", "test_oracle_pins.py") + "::test_random_walk_worked_by_hand")
    assert proc.returncode != 0
    assert "heap-buffer-overflow" in reports(log_path) and "orc_random_walk_scores" in reports(log_path)
