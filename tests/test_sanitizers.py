"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The planner (csrc/plan.cpp: a thousand lines of tile, halo and LDS arithmetic, paper section 3.2) and the
C ABI around it are built as a host program with the device launchers stubbed out, fed every workload the
test suites use plus the plans that must be rejected, and have to finish without a sanitizer report.
The oracle's C loops get the same treatment on exactly-sized buffers.
"""
import os
import subprocess

import pytest

import xl_workloads as W
from paper_2007_06000_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "paper_2007_06000_amd", "_build")
CLANG = "/opt/rocm/llvm/bin/clang++"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def dump(wl, expect=0, **options):
    opt = B.xl_options(**options)
    o = [getattr(opt, name) for name, _ in B.xl_options._fields_]
    lines = [f"workload {wl.name.replace(' ', '_')} {expect} {len(wl.layers)} {len(wl.shapes)} {len(wl.groups)} " + " ".join(map(str, o))]
    for s in wl.shapes:
        lines.append("shape " + " ".join(map(str, s)))
    for i, ly in enumerate(wl.layers):
        ins = list(ly.inputs) + [-1, -1]
        conv = ly.op == "conv"
        lines.append("layer " + " ".join(map(str, [
            B.OPS[ly.op], ins[0], ins[1], ly.out, ly.cin, ly.cout, ly.k, ly.stride, ly.pad, ly.groups, int(ly.relu),
            3 * i if conv else -1, 3 * i + 1 if conv and ly.bn else -1, 3 * i + 2 if conv and (ly.bn or ly.bias) else -1])))
    for g in wl.groups:
        lines.append(f"group {B.MODES[g.mode]} {len(g.layers)} " + " ".join(map(str, g.layers)))
    return "\n".join(lines) + "\n"


def workloads():
    text = []
    for cfg in (1, 2, 3, 4, 5):
        text.append(dump(W.config(cfg)))
        text.append(dump(W.config(cfg), precision=1))
    text.append(dump(W.config(5, n=1)))
    text.append(dump(W.config(5, n=2, hw=63, classes=40)))
    text.append(dump(W.config(3, n=0)))
    text.append(dump(W.config(4), force_tile_h=14, force_tile_w=14))
    text.append(dump(W.config(4), lds_budget_bytes=100 * 1024))
    text.append(dump(W.config(4), B.XL_E_LDS_BUDGET, lds_budget_bytes=16 * 1024))
    text.append(dump(W.config(3), paper_tuner_only=1))
    text.append(dump(W.config(3, n=1, hw=13, cin=64, s=32, e=128), force_cout_split=4))
    text.append(dump(W.config(1), force_threads=256))
    for wl in (W.straight_generic(32, 192, 28, 28, 16, 1, 0, 1, 32, 5, 2, 1), W.depthwise_pointwise(32, 16, 80, 80, 16),
               W.merge_two_producers(32), W.split_fire_pool(), W.split_fire_pool(n=3, cin=64, hw=55, s=16, e=64),
               W.conv_pool_generic(3, 3, 37, 41, 24, 3, 0, 2, 3, 2, 0), W.conv_pool_generic(2, 8, 19, 23, 40, 3, 1, 1, 3, 2, 1, bn=True),
               W.conv_gap_generic(3, 40, 13, 13, 100, 1, 0, 1), W.single_conv(1, 1, 1, 1, 1, 1),
               W.single_conv(1, 3, 17, 17, 8, 5, stride=2, pad=2), W.straight_generic(1, 3, 3, 3, 5, 3, 1, 1, 4, 3, 1, 1),
               W.config(3, n=1, hw=1, cin=8, s=16, e=32), W.config(4, n=1, hw=2, c=16), W.merge_residual_projection()):
        text.append(dump(wl))
        text.append(dump(wl, precision=1))
    # plans that must be rejected
    text.append(dump(W.merge_residual_projection(shortcut_first=False), B.XL_E_UNSUPPORTED))
    bad = W.single_conv(1, 8, 9, 9, 8, 3, pad=1)
    bad.layers[0].groups = 2
    text.append(dump(bad, B.XL_E_UNSUPPORTED))
    bad = W.config(1)
    bad.shapes[1] = (1, 16, 15, 16)
    text.append(dump(bad, B.XL_E_SHAPE))
    bad = W.config(3)
    bad.groups[0] = W.Group("merge", bad.groups[0].layers)
    text.append(dump(bad, B.XL_E_GRAPH))
    bad = W.config(4)
    bad.layers[0].inputs = (7,)
    text.append(dump(bad, B.XL_E_GRAPH))
    return "".join(text)


def test_planner_and_c_abi_under_address_and_undefined_behaviour_sanitizers():
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with sanitizer runtimes in this image")
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "planner_asan")
    csrc = os.path.join(ROOT, "paper_2007_06000_amd", "csrc")
    cmd = [CLANG, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           "-I" + csrc, "-Wno-unused-value", *SAN, os.path.join(csrc, "plan.cpp"), os.path.join(csrc, "api.cpp"),
           os.path.join(HERE, "planner_asan.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], input=workloads(), capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    assert " 0 failures" in r.stdout.splitlines()[-1]


def test_oracle_loops_under_address_and_undefined_behaviour_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_asan")
    cmd = ["gcc", "-std=c11", "-fopenmp", *SAN, os.path.join(ROOT, "oracle", "xlo.c"), os.path.join(HERE, "oracle_asan.c"),
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=0"),
                       timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
