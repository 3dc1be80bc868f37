"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the C
source is rebuilt with -fsanitize=address,undefined together with a small driver that calls every
entry point on ragged segment lists with exactly sized buffers."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_selftest")
    src = [os.path.join(ROOT, "oracle", f) for f in ("sanitize_selftest.c", "qadam_oracle.c")]
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", exe, *src, "-lm"])
    env = dict(os.environ)
    # verify_asan_link_order=0: other preloaded libraries may come before the sanitizer runtime
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "no findings" in out.stdout
