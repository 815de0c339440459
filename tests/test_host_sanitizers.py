"""The host-only sources of the library (offline compression, pattern search, test
hooks) under AddressSanitizer and UndefinedBehaviorSanitizer: a g++ build of their
own, loaded by a child process that has the sanitizer runtime preloaded and runs a
few hundred seeded compress / decompress / search cases (banded masks, empty groups,
far-apart bands, K = 1, every V, both operand formats, refused patterns).  No GPU."""
import os
import subprocess
import sys

from paper_2203_05016_amd import build as lib_build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_sources_are_clean_under_asan_and_ubsan():
    lib, runtime = lib_build.build_host_sanitized()
    env = dict(os.environ)
    # the sanitizer runtime must come first; whatever is preloaded already stays in the list
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    r = subprocess.run([sys.executable, os.path.join(HERE, "host_sanitizer_cases.py"), lib],
                       env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=600)
    out, err = r.stdout.decode(), r.stderr.decode()
    assert r.returncode == 0, "exit %d\n%s\n%s" % (r.returncode, out[-2000:], err[-4000:])
    assert "ok: 340 compress/decompress round trips, 60 searches" in out, out
    assert "ERROR: AddressSanitizer" not in err and "runtime error" not in err, err[-4000:]
