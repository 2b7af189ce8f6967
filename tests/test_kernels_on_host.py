"""The depthwise-convolution and attention kernels run on the host, thread by thread, under the address
and undefined-behaviour sanitizers: every global and LDS access of launch geometries like the GPU tests'
is checked against exactly sized buffers, and the results against float64 loops in the drivers.  The
kernels' source is taken as it is (HIP headers replaced by a small vocabulary header, launchers cut off)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2203_15952_amd", "csrc")


def spliced_source():
    src = open(os.path.join(CSRC, "conv.hip")).read()
    epi = open(os.path.join(CSRC, "epilogue.h")).read()
    epi = epi.replace("#include <hip/hip_runtime.h>", "").replace("#pragma once", "")
    assert '#include "aqt_internal.h"' in src and '#include "epilogue.h"' in src
    src = src.replace('#include "aqt_internal.h"', '#include "hip_on_host.h"').replace('#include "epilogue.h"', epi)
    assert src.count("extern __shared__ float lds[];") == 2
    src = src.replace("extern __shared__ float lds[];", "AQT_EXTERN_LDS(lds);")
    src = src[:src.index("aqt_status launch_corr")]          # kernels and geometry helpers only
    return src + open(os.path.join(HERE, "host_emulation", "conv_driver.cpp")).read()


def spliced_attention_source(driver="attention_driver.cpp"):
    src = open(os.path.join(CSRC, "attention.hip")).read()
    src = src.replace('#include "aqt_internal.h"', '#include "hip_on_host.h"')
    vec = "typedef float v4f __attribute__((ext_vector_type(4)));"      # a clang extension; g++ gets a plain struct
    assert vec in src
    src = src.replace(vec, "struct alignas(16) v4f { float x, y, z, w; };")
    vec16 = "typedef float v16f __attribute__((ext_vector_type(16)));"                # the shim has its own
    assert vec16 in src
    src = src.replace(vec16, "")
    src = src[:src.index("}  // namespace\n\nbool attention_shape_ok")]  # kernel and geometry helper only
    return src + open(os.path.join(HERE, "host_emulation", driver)).read()


def test_conv_kernels_in_bounds_and_correct_on_host(tmp_path):
    build_and_run(tmp_path, "conv_on_host", spliced_source())


def test_attention_kernel_in_bounds_and_correct_on_host(tmp_path):
    build_and_run(tmp_path, "attention_on_host", spliced_attention_source())


def test_attention_backward_kernels_in_bounds_and_correct_on_host(tmp_path):
    build_and_run(tmp_path, "attention_bwd_on_host", spliced_attention_source("attention_bwd_driver.cpp"))


def build_and_run(tmp_path, name, source):
    cpp = tmp_path / (name + ".cpp")
    cpp.write_text(source)
    exe = tmp_path / name
    cmd = ["g++", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-static-libubsan", "-std=c++20", "-pthread", "-I", os.path.join(HERE, "host_emulation"), str(cpp), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.stdout[-2000:], r.stderr[-3000:])
