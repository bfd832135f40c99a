"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer: the planner (csrc/plan.cpp has
no GPU code in it) and the C oracle are compiled with gcc's sanitizers into a small driver that
plans 1500 random chains under both objectives through the C ABI, compares them with the
oracle's exhaustive search and walks the error paths (tests/sanitizer_driver.cpp)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_and_oracle_under_asan_and_ubsan(tmp_path):
    # (the sanitizer runtimes are linked statically, so whatever the environment preloads into
    # every process does not disturb their start-up order)
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1",
           "-static-libasan", "-static-libubsan"]
    oracle_o, exe = str(tmp_path / "oracle.o"), str(tmp_path / "driver")
    subprocess.run(["gcc", "-std=c11", "-c", *san, os.path.join(ROOT, "oracle", "oracle.c"), "-o", oracle_o], check=True)
    # mom_chain_eval and the other device entry points live in eval.hip; the driver only reaches
    # their argument checks, so a stub that repeats the first of them stands in at link time
    stub = tmp_path / "stub.cpp"
    stub.write_text('#include "%s"\nextern "C" mom_status_t mom_chain_eval(const mom_plan_t *plan, const float *const *, '
                    'const int64_t *, float *d_out, int64_t, void *, size_t, uint32_t, void *)\n'
                    '{ return (!plan || !d_out) ? MOM_ERR_NULL : MOM_ERR_HIP; }\n' % os.path.join(ROOT, "include", "mom.h"))
    subprocess.run(["g++", "-std=c++17", *san, os.path.join(ROOT, "tests", "sanitizer_driver.cpp"),
                    os.path.join(ROOT, "paper_2208_10391_amd", "csrc", "plan.cpp"), str(stub), oracle_o, "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ok (0 failures)" in r.stdout
