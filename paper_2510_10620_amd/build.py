"""Builds libdcp_attn.so (HIP for gfx950 + host C++) in-tree with hipcc.

    python -m paper_2510_10620_amd.build [--force]

Objects go to paper_2510_10620_amd/_build/, the library to paper_2510_10620_amd/libdcp_attn.so.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdcp_attn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-result", "-Wno-unknown-warning-option"]


# Per-file instruction-scheduling strategy of the AMDGPU backend, chosen by measurement on MI355X: the dQ kernel gains
# 2-3 % from iterative-ilp, the dK/dV variant for tables with per-token ranges up to 3 % from max-ilp (without it the
# variant for NONE / CAUSAL tables is 1.5 % faster); the forward is best with the default.
PER_FILE_FLAGS = {
    "kernels_mfma_dkv_ranges.hip": ["-mllvm", "-amdgpu-sched-strategy=max-ilp"],
    "kernels_mfma_dq.hip": ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"],
}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "dcp.h"))
    return hs


def _compile(src, force):
    obj = os.path.join(BUILD, src + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path] + headers())
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj, False
    cmd = [HIPCC] + COMMON + PER_FILE_FLAGS.get(src, []) + ["-x", "hip", "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn.strip():
        sys.stderr.write(warn + "\n")
    return obj, True


def build_variant(out_path, defines, extra_flags=()):
    """Builds the library with extra -D flags into another file (for kernel experiments)."""
    import tempfile
    tmp = tempfile.mkdtemp(prefix="dcp_variant_")
    objs = []
    for src in sources():
        obj = os.path.join(tmp, src + ".o")
        cmd = ([HIPCC] + COMMON + PER_FILE_FLAGS.get(src, []) + list(extra_flags) + ["-D" + d for d in defines]
               + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(r.stderr)
        objs.append(obj)
    r = subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out_path] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr)
    return out_path


def build(force=False, verbose=True):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        res = list(ex.map(lambda s: _compile(s, force), sources()))
    objs = [o for o, _ in res]
    if force or any(ch for _, ch in res) or not os.path.exists(LIB):
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
