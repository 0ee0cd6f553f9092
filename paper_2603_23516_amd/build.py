"""Compile the HIP sources for gfx950 into in-tree shared libraries (hipcc cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]

LIBMSA = os.path.join(HERE, "libmsa.so")
LIBMSA_SRC = [os.path.join(HERE, "csrc", f) for f in
              ("msa_api.hip", "msa_build.hip", "msa_pool.hip", "msa_score.hip", "msa_score_gemm.hip", "msa_attend.hip", "msa_attend_prefill.hip", "msa_fetch.hip")]
LIBSYNTH = os.path.join(ROOT, "msa_synth", "libmsa_synth.so")
LIBSYNTH_SRC = [os.path.join(ROOT, "msa_synth", "csrc", "synth_fill.hip")]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    if res.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + "\n".join(lines))
    return "\n".join(lines)


def build_all(verbose=False):
    """Compile libmsa.so (the product) and libmsa_synth.so (the input generator's device fill)."""
    out = _run([HIPCC] + COMMON + ["-I", os.path.join(ROOT, "include")] + LIBMSA_SRC + ["-o", LIBMSA])
    out += _run([HIPCC] + COMMON + LIBSYNTH_SRC + ["-o", LIBSYNTH])
    if verbose and out.strip():
        print(out)
    return [LIBMSA, LIBSYNTH]


if __name__ == "__main__":
    print("\n".join(build_all(verbose=True)))
