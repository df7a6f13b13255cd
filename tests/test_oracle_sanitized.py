"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the hand-worked
case, the empty-segment case, the fixed-budget, pinned-cluster, cache-build and k-means pins run again in a child
process that loads a sanitized build of oracle/dp_oracle.c; any out-of-bounds access, use of uninitialised stack
or undefined arithmetic there aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PINS = ("hand_case or empty_segment or fixed_budget or budget_step or pinned or build_cluster_cache or rebuilt_cache "
        "or kmeans or brute_force or inclusive or group_union_with_one_head")


def test_oracle_pins_pass_under_address_and_ub_sanitizers(tmp_path):
    import oracle
    lib = oracle.build_sanitized(str(tmp_path / "libdp_oracle_asan.so"))
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's libasan.so not found"
    env = dict(os.environ)
    # the sanitizer runtime has to be the first preloaded library of the python process; whatever is preloaded
    # already stays behind it
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["DP_ORACLE_LIB"] = lib
    env["OMP_NUM_THREADS"] = "2"
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-q", "-x",
                          "-p", "no:cacheprovider", "-k", PINS], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=600)
    tail = res.stdout[-4000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
