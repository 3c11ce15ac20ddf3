"""CPU replay of the hand-counted vector-memory bookkeeping of the pipelined pointwise tile.

csrc/pw_pipe_body.hpp issues its loads through inline assembly and waits with counts it keeps
itself; a count that is too large lets a wave use data that has not landed, or end with loads in
flight.  Nothing on the GPU reports that.  Here the very same tile function is compiled for the
host (tests/sim/pw_pipe_sim_shim.hpp stands in for the loads, waits, barriers and compiler
builtins), run lane by lane for every workgroup of small launches, and the recorded request /
wait / use streams are replayed under in-order completion with the latest completion the waits
allow (tests/sim/pw_pipe_sim_main.cpp lists what is checked).  Built with AddressSanitizer, so a
plain LDS access outside the workgroup's allocation is caught too.
"""
import os
import re
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2103_16827_amd", "csrc")
SIM = os.path.join(HERE, "sim")
CLANG = "/opt/rocm/llvm/bin/clang++"


def generate(tmp, mutate=None):
    """The tile's source without its two device-only includes, and ConvParams as common.hpp has it."""
    body = open(os.path.join(CSRC, "pw_pipe_body.hpp")).read()
    body = body.replace('#include "common.hpp"\n', "").replace('#include "vmem.hpp"\n', "")
    assert "common.hpp" not in body.split("namespace qasr")[0]
    if mutate:
        body = mutate(body)
    open(os.path.join(tmp, "pw_pipe_body_stripped.hpp"), "w").write(body)
    common = open(os.path.join(CSRC, "common.hpp")).read()
    m = re.search(r"struct ConvParams \{.*?\n\};", common, flags=re.S)
    assert m, "ConvParams not found in common.hpp"
    open(os.path.join(tmp, "conv_params_extract.hpp"), "w").write(
        "#pragma once\n#include <cstdint>\nnamespace qasr {\n" + m.group(0) + "\n}\n")


def build_and_run(tmp, small=False):
    exe = os.path.join(tmp, "pw_pipe_sim")
    cmd = [CLANG, "-std=c++17", "-O0", "-g0", "-fsanitize=address,undefined", "-fno-sanitize=shift", "-fno-sanitize-recover=all",
           "-Wno-unknown-attributes", "-Wno-ignored-attributes", "-I", tmp, "-I", SIM,
           os.path.join(SIM, "pw_pipe_sim_main.cpp"), "-o", exe] + (["-DSIM_SMALL"] if small else [])
    c = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert c.returncode == 0, c.stderr[-6000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1")
    return subprocess.run([exe], capture_output=True, text=True, timeout=900, env=env)


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no host clang beside the HIP toolchain")
def test_request_bookkeeping_of_the_pointwise_tile_replays_cleanly(tmp_path):
    generate(str(tmp_path))
    r = build_and_run(str(tmp_path))
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "all cases passed" in r.stdout
    assert r.stdout.count("\nok ") + r.stdout.startswith("ok ") >= 11


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no host clang beside the HIP toolchain")
@pytest.mark.parametrize("what", ["wait_too_short", "no_final_drain", "residual_rows_too_early"])
def test_the_replay_catches_planted_mistakes(tmp_path, what):
    """The same replay on a copy of the source with a mistake planted in it (on the CPU only): a
    wait in the chunk loop that allows one request too many, a tile that returns without its final
    drain, and the lean form's residual rows sent into activation chunks that are still being read."""
    def mutate(body):
        if what == "wait_too_short":
            a = "wait_vm<(LOOK - 1) * NT>();"
            assert a in body
            return body.replace(a, "wait_vm<(LOOK - 1) * NT + 1>();")
        if what == "residual_rows_too_early":
            a = "constexpr int kLeanResAfter = 5;"
            assert a in body
            return body.replace(a, "constexpr int kLeanResAfter = 2;")
        a = "  wait_vm<0>();\n#pragma unroll\n  for (int h = 0; h < LOOK; ++h)"
        assert a in body
        return body.replace(a, "#pragma unroll\n  for (int h = 0; h < LOOK; ++h)")
    generate(str(tmp_path), mutate)
    r = build_and_run(str(tmp_path), small=True)
    assert r.returncode != 0 and "SIM FAILURE" in r.stderr, (r.stdout[-2000:], r.stderr[-2000:])


# ---- the pipelined depthwise kernel, replayed the same way

def generate_dw(tmp, mutate=None):
    """dw_pipe.hip from its namespace to the end of the planner (kernel, geometry, plan), without
    the includes and the launch code; the kernel's dynamic LDS is the simulated allocation and its
    one read of loaded rows goes through the recording stand-in."""
    src = open(os.path.join(CSRC, "dw_pipe.hip")).read()
    a = src.index("namespace qasr {")
    b = src.index("template <int KC, int R, int NI>\nhipError_t launch_t")
    body = src[a:b] + "\n}  // namespace\n}  // namespace qasr\n"
    ext = "  extern __shared__ __align__(16) unsigned char strips_lds[];"
    assert ext in body
    body = body.replace(ext, "  unsigned char* const strips_lds = sim::S().lds;  ")
    rd = "*reinterpret_cast<const v4i*>(rows_lds + lds_off[2 * q + e] + kc * 64)"
    assert rd in body
    body = body.replace(rd, "sim_lds_read16(rows_lds + lds_off[2 * q + e] + kc * 64)")
    if mutate:
        body = mutate(body)
    open(os.path.join(tmp, "dw_pipe_stripped.hpp"), "w").write("#include <type_traits>\n" + body)
    generate(tmp)          # (ConvParams)


def build_and_run_dw(tmp):
    exe = os.path.join(tmp, "dw_pipe_sim")
    cmd = [CLANG, "-std=c++17", "-O0", "-g0", "-fsanitize=address,undefined", "-fno-sanitize=shift",
           "-fno-sanitize-recover=all", "-Wno-unknown-attributes", "-Wno-ignored-attributes", "-I", tmp, "-I", SIM,
           os.path.join(SIM, "dw_pipe_sim_main.cpp"), "-o", exe]
    c = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert c.returncode == 0, c.stderr[-6000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1")
    return subprocess.run([exe], capture_output=True, text=True, timeout=900, env=env)


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no host clang beside the HIP toolchain")
def test_request_bookkeeping_of_the_depthwise_kernel_replays_cleanly(tmp_path):
    generate_dw(str(tmp_path))
    r = build_and_run_dw(str(tmp_path))
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "all cases passed" in r.stdout


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no host clang beside the HIP toolchain")
@pytest.mark.parametrize("what", ["rows_wait_too_short", "constants_not_waited_for"])
def test_the_depthwise_replay_catches_planted_mistakes(tmp_path, what):
    def mutate(body):
        if what == "rows_wait_too_short":
            a = "wait_vm_dyn(2 * L + min(it, 2) * 2 * NP);"
            assert a in body
            return body.replace(a, "wait_vm_dyn(2 * L + min(it, 2) * 2 * NP + 1);")
        a = "  wait_vm_dyn(n_rows);                          // everything requested before the rows is here"
        assert a in body
        return body.replace(a, "  wait_vm_dyn(n_rows + 2);")
    generate_dw(str(tmp_path), mutate)
    r = build_and_run_dw(str(tmp_path))
    assert r.returncode != 0 and "SIM FAILURE" in r.stderr, (r.stdout[-2000:], r.stderr[-2000:])
