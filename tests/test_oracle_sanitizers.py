"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The oracle is what every parity claim rests on, so its own memory accesses and arithmetic are checked with
instrumented code: the pins of the worked example (Fig. 2), the brute-force and LP comparisons, the rounding
definition with its tie-breaks, the adversarial local-search case and the early-exit variant run in a child
process that loads a build of oracle/tsenor_oracle.c with -fsanitize=address,undefined (any report aborts).
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PINS = ("fig2 or brute_force or exact_solvers or lp_optimum or rounding_matches or adversarial or tie_break "
        "or early_exit or simple_rounding or objective_packing or large_logits or composed_path")


def test_oracle_pins_pass_under_asan_and_ubsan():
    sys.path.insert(0, ROOT)
    import oracle

    lib = oracle.build_sanitized()
    runtimes = [subprocess.run(["gcc", f"-print-file-name={n}"], capture_output=True, text=True, check=True).stdout.strip()
                for n in ("libasan.so", "libubsan.so")]
    assert all(os.path.isabs(r) and os.path.exists(r) for r in runtimes), runtimes
    env = dict(os.environ)
    # the sanitizer runtime has to come first in the child's library list; whatever was preloaded stays behind it
    env["LD_PRELOAD"] = ":".join(runtimes + [x for x in env.get("LD_PRELOAD", "").split(":") if x])
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"      # (the interpreter itself leaks)
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["TSENOR_ORACLE_LIBRARY"] = str(lib)
    env["OMP_NUM_THREADS"] = "4"
    check = ("import oracle, sys; p = oracle.loaded_library(); print('oracle library:', p); "
             "sys.exit(0 if p.endswith('libtsenor_oracle_sanitized.so') else 3)")
    r = subprocess.run([sys.executable, "-c", check], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join("tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider", "-k", PINS],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
    passed = int(r.stdout.strip().splitlines()[-1].split(" passed")[0].split()[-1])
    assert passed >= 15, tail
