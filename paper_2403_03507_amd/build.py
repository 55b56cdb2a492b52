"""Build libgalore.so (gfx950) in-tree with hipcc: one object per csrc/*.hip, compiled in parallel, plus a check
of the compiler's assembly output that the hand-counted wait of the weight-update GEMM relies on."""
import concurrent.futures
import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgalore.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + os.environ.get("GALORE_HIPCC_EXTRA", "").split()


def _compile(src):
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", src, "-o", obj]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def check_weight_prefetch_assembly():
    """The weight-update kernel lets its early W prefetch stay in flight across one barrier with
    `s_waitcnt vmcnt(8)`: right only if the compiler emits exactly 8 vector-memory loads for the 8 prefetched
    slices, after the 8 tile loads of the same K step and with no store in between.  A compiler that merged,
    split or moved those loads would make the kernel read stale weights without any error, so the library is
    not built unless the device assembly of gemm_bf16.hip has that shape in all three weight-update kernels
    ((K,X), (K,K), and (K,K) for W of any alignment).  Raises RuntimeError otherwise."""
    src = os.path.join(CSRC, "gemm_bf16.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm_bf16.s")
        p = subprocess.run([HIPCC] + [f for f in FLAGS if f != "-fPIC"] + ["-S", "--cuda-device-only", "-o", out, src],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if p.returncode != 0:
            raise RuntimeError("hipcc -S failed on %s:\n%s" % (src, p.stdout))
        text = open(out).read()
    kernels = re.findall(r"^(_ZN6galore14gemm_dl_kernelILb1ELb[01]ELNS_8EpilogueE1E\w+):[^\n]*\n(.*?)\.end_amdhsa_kernel", text,
                         flags=re.S | re.M)
    if len(kernels) != 3 or sum(name.endswith("Lb1EEEvNS_9GemmGroupE") for name, _ in kernels) != 1:
        raise RuntimeError("expected the three weight-update kernels in the assembly of gemm_bf16.hip, found %d" % len(kernels))
    for name, body in kernels:
        ops = []
        for line in body.split("\n"):
            t = line.split(";")[0].strip()
            if t.startswith("global_load_lds"):
                ops.append("T")                                 # tile load (direct to LDS)
            elif t.startswith("global_load"):
                ops.append("W")                                 # load into registers: the W prefetch
            elif t.startswith("global_store") or t.startswith("global_atomic"):
                ops.append("S")
            elif t.startswith("s_waitcnt") and "vmcnt(8)" in t:
                ops.append("8")
            elif t.startswith("s_barrier"):
                ops.append("B")
        seq = "".join(ops)
        if "8" not in seq:
            raise RuntimeError("%s: no s_waitcnt vmcnt(8)" % name)
        first = seq.index("8")      # the hand-written wait; the compiler's own waits for the prefetched registers come later
        before = seq[:first]
        ok = (seq[first + 1:first + 2] == "B" and before.endswith("T" * 8 + "W" * 8) and "B" in before
              and "S" not in before[before.rindex("B"):])
        if not ok:
            raise RuntimeError("%s: the early W prefetch is not 8 tile loads followed by exactly 8 register loads before "
                               "the vmcnt(8) wait and its barrier (tail of the sequence: %s)" % (name, before[-40:]))
    return len(kernels)


def build(verbose=False):
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
        check = ex.submit(check_weight_prefetch_assembly)
        objs = list(ex.map(_compile, srcs))
        check.result()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
