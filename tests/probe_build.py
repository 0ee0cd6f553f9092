"""Builds the test-only probe library (tests/csrc/probe.hip: small kernels that pin the device-side layout
assumptions -- MFMA operand order, DPP patterns, global -> LDS copies, key packing -- the parity tests rest on)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIBPROBE = os.path.join(HERE, "libmsa_probe.so")
LIBPROBE_SRC = os.path.join(HERE, "csrc", "probe.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def build_probe(force=True):
    """Compile the probe library; with force=False only when it is missing or older than its source."""
    if not force and os.path.exists(LIBPROBE) and os.path.getmtime(LIBPROBE) >= os.path.getmtime(LIBPROBE_SRC):
        return LIBPROBE
    res = subprocess.run([HIPCC] + FLAGS + ["-I", os.path.join(os.path.dirname(HERE), "paper_2603_23516_amd", "csrc"),
                                            LIBPROBE_SRC, "-o", LIBPROBE],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("probe build failed:\n" + res.stdout)
    return LIBPROBE
