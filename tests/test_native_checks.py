"""Host-only native checks (no GPU): the oracle's C code under AddressSanitizer and
UndefinedBehaviorSanitizer, and the unit test of the launch-limit rule the library applies before
it accepts a state."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")


def _run(cmd, env=None, timeout=600):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=timeout, env=env)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-3000:]}\n{res.stderr[-3000:]}"
    return res.stdout + res.stderr


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitizer_run")
    srcs = [os.path.join(ROOT, "oracle", f) for f in ("philox.c", "classic.c", "craftax_full.c")]
    _run(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-static-libasan", "-o", exe, os.path.join(NATIVE, "oracle_sanitizer_run.c")] + srcs + ["-lm"])
    env = dict(os.environ)                          # the sanitizer runtime is linked statically: whatever is preloaded stays
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    out = _run([exe], env=env)
    assert "oracle_sanitizer_run: ok" in out and "runtime error" not in out and "AddressSanitizer" not in out, out[-3000:]


def test_regeneration_units_are_dealt_out_exactly_once(tmp_path):
    """The walk that shares the regeneration units of a step launch between its blocks (csrc/regen_units.hpp)."""
    exe = str(tmp_path / "regen_units_test")
    _run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-o", exe, os.path.join(NATIVE, "regen_units_test.cpp")])
    assert "regen_units_test: ok" in _run([exe])


def test_public_header_compiles_as_c_and_as_cpp(tmp_path):
    """include/craftax.h on its own, with warnings as errors, as C11 and as C++17: no HIP or torch type
    in any signature, every struct complete."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    body = '#include "craftax.h"\nint main(void) { craftax_config c; craftax_metrics m; (void)c; (void)m; return (int)sizeof(craftax_metrics) == 0; }\n'
    for name, cc, std in (("use.c", "gcc", "-std=c11"), ("use.cpp", "g++", "-std=c++17")):
        src = tmp_path / name
        src.write_text(body)
        _run([cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), "-c", "-o", str(tmp_path / (name + ".o")), str(src)])


def test_launch_limit_rule(tmp_path):
    exe = str(tmp_path / "launch_limits_test")
    _run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", "-o", exe, os.path.join(NATIVE, "launch_limits_test.cpp")])
    assert "launch_limits_test: ok" in _run([exe])
