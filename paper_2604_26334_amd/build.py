"""Build libpshard.so (host planner/scheduler/packer + HIP kernels and executor) for gfx950.

Besides compiling, the build CHECKS what the hand-placed waits of the MFMA GEMM rely on, from the
compiler's own output for kernels.hip, and fails if it does not hold:
  - no kernel of the matmul / attention families uses scratch memory or spills a register (a spill
    reload is a vector-memory operation and would be counted by `s_waitcnt vmcnt(n)` like a prefetch);
  - in every gemm_w4_kernel, a vmcnt(0) stands between the opening prefetches and the first barrier; every later stretch
    between two barriers that ends in a counted wait vmcnt(n > 0) issues exactly the loads of one
    prefetch, LDS fills first, and n is the count the kernel's ring depth implies; nothing else
    touches vector memory inside the ring.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ROOT = os.path.dirname(HERE)
LIB = os.environ.get("PS_LIB_OUT", os.path.join(HERE, "libpshard.so"))
BUILD = os.path.join(HERE, "_build")
SOURCES = ["planner.cpp", "schedule.cpp", "pack.cpp", "cpu_backend.cpp", "profile_db.cpp", "kernels.hip", "stack.hip", "profile.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off: results must not depend on which kernel a device function was inlined into
# (the one-token kernel variants have to agree bit for bit on every placement); fused multiply-adds
# are written out with fmaf where they are wanted
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC] + os.environ.get("PS_EXTRA_FLAGS", "").split()
CHECKED = "kernels.hip"      # the source whose kernels are checked
NO_SCRATCH = ("gemm_w4_kernel", "gemv_w4_kernel", "gemv_mt_kernel", "attn_decode_kernel", "attn_combine_kernel", "attn_chunk_kernel", "attn_chunk_mfma_kernel", "attn_chunk_onepass_kernel", "attn_combine_chunk_kernel")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), err[-4000:]))
    return r.stderr


def _compile(src):
    obj = os.path.join(BUILD, src + ".o")
    hip = ["-x", "hip"] if src.endswith(".hip") else []
    remarks = ["-Rpass-analysis=kernel-resource-usage"] if src == CHECKED else []
    err = _run([HIPCC] + FLAGS + hip + remarks + ["-c", os.path.join(CSRC, src), "-o", obj])
    if src == CHECKED:
        check_resource_usage(err)
    else:
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def _isa(src):
    """Device assembly of one HIP source (a second, device-only compile next to the object build)."""
    out = os.path.join(BUILD, src + ".s")
    _run([HIPCC] + FLAGS + ["-x", "hip", "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out])
    return out


def check_resource_usage(remarks):
    """The compiler's per-kernel resource remarks: matmul and attention kernels use no scratch, and the
    gather copy kernel holds a CU's whole LDS (what keeps matmul workgroups off the CUs it reads PCIe from)."""
    name, bad, seen, gather_lds = None, [], 0, None
    for ln in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", ln)
        if m:
            name = m.group(1)
            seen += any(k in name for k in NO_SCRATCH)
            continue
        m = re.search(r"remark:\s+LDS Size \[bytes/block\]: (\d+)", ln)
        if m and name and "h2d_gather_kernel" in name:
            gather_lds = int(m.group(1))
        m = re.search(r"remark:\s+(ScratchSize \[bytes/lane\]|SGPRs Spill|VGPRs Spill): (\d+)", ln)
        if m and name and any(k in name for k in NO_SCRATCH) and int(m.group(2)) != 0:
            bad.append("%s: %s = %s" % (name, m.group(1), m.group(2)))
    if seen == 0:
        raise RuntimeError("build check: no resource-usage remarks for the matmul kernels (compiler flag ignored?)")
    if bad:
        raise RuntimeError("build check: scratch / spills in kernels that must have none:\n  " + "\n  ".join(bad))
    if gather_lds != 160 * 1024:
        raise RuntimeError("build check: h2d_gather_kernel allocates %s B of LDS, not the CU's 163840" % gather_lds)


def gemm_wait_counts(mt, nw, at=2):
    """(loads per prefetch, LDS fills among them, counted wait of a steady step) of gemm_w4_kernel<.., at, mt, .., nw>."""
    nfill = mt // (4 * nw)
    lpi = nfill + at
    depth = 3 if nw == 8 else (2 if mt <= 64 else 1)
    early = depth >= 3
    land = depth - 2 if early else depth - 1
    return lpi, nfill, land * lpi + (at if early else 0)


def check_gemm_isa(path):
    """The invariant behind the GEMM's hand-counted waits, read off the generated code."""
    txt = open(path).read()
    funcs = re.findall(r"^(_ZN2ps14gemm_w4_kernel\w+):[^\n]*\n(.*?)\n\.Lfunc_end", txt, flags=re.S | re.M)
    if not funcs:
        raise RuntimeError("build check: no gemm_w4_kernel in " + path)
    bad = []
    for mangled, body in funcs:
        m = re.match(r"_ZN2ps14gemm_w4_kernelILi(\d+)ELi(\d+)ELi(\d+)ELb([01])ELi(\d+)EEE", mangled)
        if not m:
            bad.append(mangled + ": unexpected template arguments")
            continue
        at, mt, nw = int(m.group(2)), int(m.group(3)), int(m.group(5))
        lpi, nfill, in_flight = gemm_wait_counts(mt, nw, at)
        segs, cur = [], []
        for ln in body.splitlines():
            f = ln.split()
            if not f:
                continue
            ins = f[0]
            if ins == "s_barrier":
                segs.append(cur)
                cur = []
            elif re.match(r"(buffer_|global_|flat_|scratch_)", ins):
                cur.append("lds" if (ins.startswith("buffer_load") and re.search(r"\blds\b", ln)) else ins)
            elif ins == "s_waitcnt" and "vmcnt" in ln:
                cur.append(int(re.search(r"vmcnt\((\d+)\)", ln).group(1)))
        segs.append(cur)        # the epilogue, after the last barrier
        if any(isinstance(x, str) and (x.startswith("scratch_") or x.startswith("flat_")) for s in segs for x in s):
            bad.append(mangled + ": scratch or flat memory instruction")
        if len(segs) < 3:
            bad.append(mangled + ": no barrier-delimited ring found")
            continue
        # (waits the compiler adds behind it for its own bookkeeping change nothing)
        last_load = max([k for k, x in enumerate(segs[0]) if isinstance(x, str)], default=-1)
        if 0 not in segs[0][last_load + 1:]:
            bad.append(mangled + ": no vmcnt(0) between the opening prefetches and the first barrier")
        steps = 0
        for s in segs[1:-1]:
            loads = [x for x in s if isinstance(x, str)]
            waits = [x for x in s if isinstance(x, int)]
            if "lds" not in loads:
                continue       # not a ring step
            steps += 1
            if not waits:
                bad.append(mangled + ": ring step without a vmcnt wait")
            elif waits[-1] != 0:
                if waits[-1] != in_flight:
                    bad.append("%s: counted wait vmcnt(%d), expected %d" % (mangled, waits[-1], in_flight))
                # every prefetch: the activation fills, then one code load per tile; one prefetch in eight
                # starts with a scale fill per tile (a branch: the text holds it either way)
                nl = sum(1 for x in loads if x == "lds")
                if nl not in (nfill, nfill + at) or loads[:nl] != ["lds"] * nl or len(loads) != nl + at:
                    bad.append("%s: a counted ring step issues %s, expected (%d +) %d LDS fills then %d weight loads" % (
                        mangled, loads, at, nfill, at))
                if any(not x.startswith("buffer_load") for x in loads if x != "lds"):
                    bad.append(mangled + ": a ring step touches vector memory with something other than its prefetch")
        if steps == 0:
            bad.append(mangled + ": no ring step recognised")
    if bad:
        raise RuntimeError("build check: the GEMM's counted waits do not match the generated code:\n  " + "\n  ".join(bad))
    return len(funcs)


def build():
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        isa = ex.submit(_isa, CHECKED)
        objs = list(ex.map(_compile, SOURCES))
        n = check_gemm_isa(isa.result())
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    sys.stderr.write("build checks passed: no scratch in the matmul/attention kernels; %d GEMM instantiations match their wait counts\n" % n)
    return LIB


if __name__ == "__main__":
    print(build())
