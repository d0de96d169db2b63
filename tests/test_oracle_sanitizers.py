"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the C
source is built with -fsanitize=address,undefined and every pin of tests/oracle_pins.py runs
against that build in a child process.  A clean exit means the pins hold AND no access left
its buffer, no shift or cast was undefined, on all the ragged inputs the pins use.  Two planted
memory mistakes show that the sanitizer build really watches: each passes or fails the pins
on values alone, but must die under the sanitizer."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "ckpt_oracle.c")
PINS = os.path.join(HERE, "oracle_pins.py")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def asan_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE,
                          text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def build(src, lib):
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-w"] + SAN +
                   ["-fPIC", "-shared", "-pthread", str(src), "-o", str(lib)], check=True)


def run_pins_under_sanitizers(lib):
    """The interpreter is not instrumented, so the sanitizer runtime is put in front of the
    child's preload list (whatever that list already holds stays in it)."""
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (asan_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1"
    return subprocess.run([sys.executable, PINS, str(lib)], env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True)


@pytest.fixture(scope="module", autouse=True)
def need_toolchain():
    pytest.importorskip("xxhash")
    if asan_runtime() is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")


def test_pins_hold_and_nothing_trips_the_sanitizers(tmp_path):
    lib = tmp_path / "libckpt_oracle_san.so"
    build(SRC, lib)
    p = run_pins_under_sanitizers(lib)
    assert p.returncode == 0, p.stdout[-3000:]
    assert "ERROR: AddressSanitizer" not in p.stdout and "runtime error" not in p.stdout


@pytest.mark.parametrize("name,old,new", [
    ("compact pads one byte too many",
     "memset(out + soff + len, 0, padded - len);", "memset(out + soff + len, 0, padded - len + 1);"),
    ("restore copies far past the chunk",
     "in + m->stage_off, m->len);", "in + m->stage_off, (size_t)m->len + 100000);"),
])
def test_a_planted_overrun_dies_under_the_sanitizers(name, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) == 1, f"site for '{name}' not unique"
    src, lib = tmp_path / "overrun.c", tmp_path / "liboverrun_san.so"
    src.write_text(text.replace(old, new))
    build(src, lib)
    p = run_pins_under_sanitizers(lib)
    assert p.returncode != 0
    assert "AddressSanitizer" in p.stdout, p.stdout[-2000:]
