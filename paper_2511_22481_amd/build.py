"""Compile the HIP library for gfx950 in-tree (paper_2511_22481_amd/libomniattn.so)."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libomniattn.so")
SOURCES = ["decode_kernels.hip", "decode_fp8_kernel.hip", "append_kernels.hip", "api.cpp", "plan.cpp"]
HEADERS = ["kernels.h", "plan.h", "decode_common.h", os.path.join("..", "..", "include", "omniattn.h")]


def hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


STAMP = LIB + ".stamp"   # hash of the sources the library was built (and checked) from
CHECKER = os.path.join(HERE, "check_isa.py")


def source_hash():
    h = hashlib.sha256()
    for f in sorted(SOURCES + HEADERS):
        h.update(f.encode())
        h.update(open(os.path.join(CSRC, f), "rb").read())
    h.update(open(CHECKER, "rb").read())
    return h.hexdigest()


def is_stale():
    """True unless the library exists and was built, and its generated code checked, from
    exactly the present sources (content hash, so that file times do not matter)."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    return open(STAMP).read().strip() != source_hash()


def build(force=True, verbose=False):
    """hipcc --offload-arch=gfx950, one shared library.  Packed-fp32 code generation
    is switched off for the device pass."""
    if not force and not is_stale():
        return LIB
    if os.path.exists(STAMP):
        os.remove(STAMP)
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-x", "hip"]
    cmd += [os.path.join(CSRC, f) for f in SOURCES]
    cmd += ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines()
                        if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    check_generated_code(verbose)
    with open(STAMP, "w") as f:     # only a library whose generated code passed the check is stamped
        f.write(source_hash() + "\n")
    return LIB


def check_generated_code(verbose=False):
    """Emit the device assembly of the kernels once more and run the static hazard
    check on it (see check_isa.py); raises if compiler-inserted code reads an MFMA
    result too early."""
    import tempfile
    from .check_isa import check
    problems = []
    with tempfile.TemporaryDirectory() as tmp:
        for src, kernel in (("decode_kernels.hip", "decode_kernel"), ("decode_fp8_kernel.hip", "decode_fp8_kernel")):
            out = os.path.join(tmp, src + ".s")
            cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++20",
                   "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                   "-Wno-unused-command-line-argument", "--cuda-device-only", "-S", "-x", "hip",
                   os.path.join(CSRC, src), "-o", out]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc -S failed:\n" + res.stderr[-2000:])
            problems += check(open(out).read(), kernel)
    if problems:
        raise RuntimeError("generated code reads MFMA results too early:\n" + "\n".join(problems[:20]))
    if verbose:
        print("ISA hazard check: ok")


if __name__ == "__main__":
    import sys
    sys.path.insert(0, os.path.dirname(HERE))
    from paper_2511_22481_amd.build import build as _b
    print(_b(verbose=True))
