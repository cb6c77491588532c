"""Build libsurelock.so (HIP, gfx950 only) in-tree next to this file.

    python -m paper_2602_06412_amd.build

Each .hip under csrc/ is compiled to an object in parallel, then linked.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsurelock.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result",
         # the direct-to-LDS loads set M0 inside their asm statement and list it as clobbered on purpose
         "-Wno-inline-asm",
         # per-kernel register / scratch report, checked below for the kernels that must not spill
         "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"]

# Kernels whose correctness rests on registers the compiler must not spill or copy (operand rings filled by
# inline-assembly loads and waited for with hand-counted vmcnt): any scratch use fails the build.
NO_SCRATCH = ("gemm_stream_kernel",)


def _resource_report(out):
    """{mangled kernel name: {field: int}} from the compiler's kernel-resource-usage remarks."""
    import re
    rep, cur = {}, None
    for line in out.splitlines():
        m = re.search(r"remark: .*Function Name: (\S+)", line)
        if m:
            cur = rep.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark: .*?\s{2,}([A-Za-z][A-Za-z /\[\]]+?): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return rep


def check_no_scratch(src, out):
    for name, f in _resource_report(out).items():
        if any(k in name for k in NO_SCRATCH):
            bad = {k: v for k, v in f.items() if ("Scratch" in k or "Spill" in k) and v != 0}
            if bad or "ScratchSize [bytes/lane]" not in f:
                raise RuntimeError(f"{src}: kernel {name} must not use scratch or spill registers, compiler reports {bad or f}")


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src):
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r.returncode, r.stdout + r.stderr


def build(verbose=True, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        for src, obj, rc, out in ex.map(_compile, sources()):
            if rc != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{out}")
            check_no_scratch(src, out)
            msgs = "\n".join(l for l in out.splitlines()
                             if "packed-fp32-ops" not in l and "remark:" not in l and l.strip())
            if verbose and msgs:
                print(f"[{src}]\n{msgs}")
            objs.append(obj)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
