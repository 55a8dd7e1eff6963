"""Build libs2attn.so (HIP, gfx950) in-tree with hipcc, and check the emitted assembly of the kernels (isa_check)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libs2attn.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def build(verbose=False, extra=(), jobs=None):
    from concurrent.futures import ThreadPoolExecutor

    try:
        from . import isa_check
    except ImportError:                                # run as a script
        sys.path.insert(0, HERE)
        import isa_check

    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)

    def compile_one(s):
        o = os.path.join(HERE, "_build", os.path.basename(s) + ".o")
        cmd = ["hipcc", "-x", "hip", "-c", s, "-o", o] + [f for f in FLAGS if f != "-shared"] + list(extra)
        if s.endswith(".hip"):
            cmd.append("-save-temps=obj")          # keeps the device assembly next to the object for the check below
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        if s.endswith(".hip"):
            asm = os.path.join(HERE, "_build", os.path.basename(s)[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
            findings = isa_check.scan_file(asm)
            if findings:
                raise RuntimeError("matrix-core result read too early in " + os.path.basename(s) + ":\n" + "\n".join(findings))
        return o

    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, sources()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
