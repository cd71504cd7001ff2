"""Sanitizer tier for the CPU code: the oracle and the host build of the kernels' building blocks are compiled
with -fsanitize=address,undefined and their pins run through those builds in a child process (the sanitizer
runtime has to be loaded before the interpreter starts).  Any out-of-bounds access, use of an uninitialised
shift, signed overflow or misaligned access in them aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    out = subprocess.run(["g++", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def _child(pytest_args, timeout):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    assert asan, "g++ has no libasan.so"
    env = dict(os.environ)
    pre = [asan] + ([ubsan] if ubsan else []) + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["FCV2_ORACLE_SANITIZE"] = "1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + pytest_args,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    assert r.returncode == 0, f"sanitized run failed ({r.returncode}):\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    assert "passed" in r.stdout and "libfcv2_oracle_asan" not in r.stderr
    return r.stdout


def test_oracle_pins_under_address_and_ub_sanitizers():
    # layout, quantizer, planes, record round trips, reduce, integer metadata and dispatch pins
    out = _child(["tests/test_oracle_pins.py", "-k",
                  "layout or footprint or quantizer or planes or roundtrip or reduce or dispatch or meta_int or "
                  "spike_select_closed_form or peer_order or fused_multiply"], 600)
    assert " passed" in out


def test_kernel_building_blocks_under_address_and_ub_sanitizers():
    out = _child(["tests/test_host_logic.py", "-k",
                  "plane_packing or pair_decoding or bf16_helpers or scale_int_ends or launch_plan or short_division"], 600)
    assert " passed" in out


def test_the_sanitized_builds_are_what_the_child_loads():
    """The switch really selects the instrumented libraries (otherwise the two tests above would prove nothing)."""
    code = ("import os, oracle; oracle.lib(); m = open('/proc/self/maps').read(); "
            "assert 'libfcv2_oracle_asan.so' in m and 'libasan' in m; print('ok')")
    asan = _runtime("libasan.so")
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join([asan] + [p for p in env.get("LD_PRELOAD", "").split(":") if p])
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"
    env["FCV2_ORACLE_SANITIZE"] = "1"
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "ok" in r.stdout, r.stderr[-2000:]
