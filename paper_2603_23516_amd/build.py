"""Compile the HIP sources for gfx950 into in-tree shared libraries (hipcc cross-compiles without a GPU).

Every source becomes one object (compiled side by side, one hipcc per source) and the objects are linked into
the library; the objects live in a `_build/` folder next to this file and are rewritten by every call."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]

LIBMSA = os.path.join(HERE, "libmsa.so")
LIBMSA_SRC = [os.path.join(HERE, "csrc", f) for f in
              ("msa_api.hip", "msa_build.hip", "msa_pool.hip", "msa_score.hip", "msa_score_gemm.hip", "msa_attend.hip", "msa_attend_prefill.hip", "msa_fetch.hip")]
LIBSYNTH = os.path.join(ROOT, "msa_synth", "libmsa_synth.so")
LIBSYNTH_SRC = [os.path.join(ROOT, "msa_synth", "csrc", "synth_fill.hip")]
OBJDIR = os.path.join(HERE, "_build")


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    if res.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + "\n".join(lines))
    return "\n".join(lines)


def _compile(src):
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    out = _run([HIPCC] + COMMON + ["-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj])
    return obj, out


def build_all(verbose=False, only=None):
    """Compile libmsa.so (the product) and libmsa_synth.so (the input generator's device fill).  `only`: a list of
    source base names to recompile (the other objects are reused unless their source or a header is newer; for quick
    rebuilds by hand)."""
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = LIBMSA_SRC + LIBSYNTH_SRC
    import glob
    headers = glob.glob(os.path.join(HERE, "csrc", "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)

    def stale(src):   # no object yet, or older than its source or than any header
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        return not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header)
    todo = [s for s in srcs if only is None or os.path.basename(s) in only or stale(s)]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        done = dict(zip(todo, ex.map(_compile, todo)))
    out = "".join(o for _, o in done.values())
    objs = {s: os.path.join(OBJDIR, os.path.basename(s) + ".o") for s in srcs}
    out += _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [objs[s] for s in LIBMSA_SRC] + ["-o", LIBMSA])
    out += _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [objs[s] for s in LIBSYNTH_SRC] + ["-o", LIBSYNTH])
    if verbose and out.strip():
        print(out)
    return [LIBMSA, LIBSYNTH]


if __name__ == "__main__":
    import sys
    print("\n".join(build_all(verbose=True, only=sys.argv[1:] or None)))
