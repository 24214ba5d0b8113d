"""The oracle and a C harness that drives every oracle function on ragged shapes, compiled with
AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU involved).  The run must
end cleanly, and its checksums must equal those of the ordinary build used by every other test."""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HARNESS = os.path.join(ROOT, "tests", "sanitize", "oracle_harness.c")
ORACLE = os.path.join(ROOT, "oracle", "rbe_oracle.c")


def build(tmp_path, flags, name):
    exe = str(tmp_path / name)
    subprocess.check_call(["gcc", "-O1", "-g", "-Wall", "-Wextra", "-Werror", *flags, "-o", exe, HARNESS, ORACLE, "-lm"])
    return exe


def run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env.pop("LD_PRELOAD", None)       # the sanitizer runtime has to come first in the process
    p = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert p.returncode == 0, f"exit {p.returncode}\n{p.stdout[-2000:]}\n{p.stderr[-4000:]}"
    assert p.stdout.strip().endswith("done")
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr[-4000:]
    return re.findall(r"^case (.*) checksum=(\S+)$", p.stdout, flags=re.M)


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    san = run(build(tmp_path, ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"], "orc_san"))
    plain = run(build(tmp_path, ["-O2"], "orc_plain"))
    assert len(san) == 7 and [c for c, _ in san] == [c for c, _ in plain]
    for (case, a), (_, b) in zip(san, plain):
        assert a == b, f"{case}: sanitized build {a} != ordinary build {b}"
