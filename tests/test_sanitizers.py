"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; GPU code cannot be
sanitized on the test machines):
  * the oracle (oracle/rd_oracle.c, gcc -fsanitize=address,undefined) runs its own pins;
  * the library's host code -- argument checks, launch plans, workspace sizing -- (host pass only,
    clang -fsanitize=address,undefined) runs the C ABI's argument-error cases, none of which launches.
Each runs in a child process that has the matching sanitizer runtime preloaded; a report from either
sanitizer makes the child fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.dirname(os.path.abspath(__file__))


def _run(tests, env_extra, preload, tmp):
    env = dict(os.environ)
    env.update(env_extra)
    prior = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = preload + (":" + prior if prior else "")          # the sanitizer runtime has to come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["HIP_VISIBLE_DEVICES"] = "-1"                                     # no device: nothing here launches anything
    env["ROCR_VISIBLE_DEVICES"] = "-1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *tests],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    return r.stdout


def test_oracle_pins_under_asan_ubsan(tmp_path):
    import oracle
    lib = oracle.build_sanitized(str(tmp_path))
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.exists(rt), rt
    tests = [os.path.join(HERE, t) for t in ("test_oracle_dedup.py", "test_oracle_attn.py", "test_oracle_accept.py",
                                             "test_oracle_commit.py", "test_oracle_rope.py", "test_oracle_draft.py",
                                             "test_oracle_accept_sample.py")]
    out = _run(tests, {"RD_ORACLE_LIB": lib}, rt, tmp_path)
    assert " passed" in out


def test_library_host_code_under_asan_ubsan(tmp_path):
    from paper_2403_09919_amd import build as rd_build
    lib, rt = rd_build.build_host_sanitized(str(tmp_path))
    assert os.path.exists(lib) and os.path.exists(rt), (lib, rt)
    out = _run([os.path.join(HERE, "test_abi.py")], {"RD_TEST_LIB": lib}, rt, tmp_path)
    assert " passed" in out
