"""Compile the HIP sources under csrc/ into paper_2511_09987_amd/libcyclotron_mm.so (gfx950 only)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcyclotron_mm.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-inline-asm",
         "-Wno-unused-command-line-argument",
         # keep hipcc from forming packed fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def reads_lds_from_asm(src: str) -> bool:
    """Does this source issue LDS reads from inline asm (their registers are valid only after a later wait)?"""
    with open(src) as f:
        return 'asm volatile("ds_read' in f.read()


def check_async_reads(src: str) -> None:
    """Compile src to assembly with the flags of the build and run check_async_reads.violations on it."""
    import importlib.util
    import tempfile
    spec = importlib.util.spec_from_file_location("check_async_reads", os.path.join(HERE, "check_async_reads.py"))
    checker = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(checker)
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "device.s")
        p = subprocess.run(["hipcc", *FLAGS, "-S", "--cuda-device-only", src, "-o", asm],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src}:\n{p.stdout}")
        with open(asm) as f:
            found = checker.violations(f.read())
    if found:
        raise RuntimeError(f"{src}: the compiler touches registers of LDS reads that are still outstanding:\n" +
                           "\n".join(found[:20]))


def build(verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Always recompiles."""
    objs = []
    procs = []
    for src in sources():
        obj = os.path.join(CSRC, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen(["hipcc", *FLAGS, "-c", src, "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    for src in sources():
        if reads_lds_from_asm(src):
            check_async_reads(src)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
