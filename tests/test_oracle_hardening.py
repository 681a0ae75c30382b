"""The checker checked: the oracle's C source built with the address and undefined-behaviour sanitizers runs
every pin (plain decode and pre-filling, chunk cache, append, FP8 storage) without a report.  Its buffers are
sized and indexed by hand per (batch, KV head) unit; a read or write past one of them, a signed overflow in an
index, or a misaligned access would otherwise only show up as a wrong number, or not at all.  CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "shadowkv_oracle.c")
PINS = ["test_oracle_pins.py", "test_oracle_cache.py", "test_oracle_append.py", "test_oracle_fp8.py",
        "test_oracle_planted.py"]


def _run_pins(tmp_path, source_text, pins):
    c_file, so_file = tmp_path / "oracle_san.c", tmp_path / "liboracle_san.so"
    c_file.write_text(source_text)
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-fno-omit-frame-pointer", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so_file), str(c_file),
                    "-lm"], check=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, stdout=subprocess.PIPE,
                          text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc has no address-sanitizer runtime here"
    # the interpreter is not instrumented: the runtime has to be loaded ahead of it.  Leak reports are off (the
    # interpreter and its extension modules never free everything); whatever else was preloaded stays.
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    env = dict(os.environ, SHADOWKV_ORACLE_LIB=str(so_file), LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=1:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    return subprocess.run([sys.executable, "-m", "pytest"] + [os.path.join(ROOT, "tests", p) for p in pins] +
                          ["-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True)


def test_pins_pass_on_a_sanitizer_build_of_the_oracle(tmp_path):
    res = _run_pins(tmp_path, open(SRC).read(), PINS)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "passed" in res.stdout and "AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout


def test_the_sanitizer_route_reports_a_planted_overrun(tmp_path):
    """The same route with one chunk logit written one element past the end of its buffer: a mistake no pin
    need notice by value (the slot is never read) has to end the run."""
    text = open(SRC).read()
    old = "P[g * n_c + j] = dot * scale;"
    assert text.count(old) == 1
    bad = text.replace(old, "P[g * n_c + j + (g == G - 1 && j == n_c - 1 ? 1 : 0)] = dot * scale;")
    res = _run_pins(tmp_path, bad, ["test_oracle_pins.py"])
    # (the report itself goes to a descriptor the test runner has captured and dies with; the abort is what shows)
    assert res.returncode in (-6, 134) and "Aborted" in res.stdout, (res.returncode, res.stdout[-2000:])
