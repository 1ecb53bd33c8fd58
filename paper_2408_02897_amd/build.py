"""Build libqmm.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2408_02897_amd.build [--force]
    python -m paper_2408_02897_amd.build --check-asm     # scan the GEMM kernels' assembly (a few minutes)
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqmm.so")
SOURCES = ["qmm_api.hip", "qmm_scale.hip", "qmm_quantize.hip", "qmm_metric.hip", "qmm_gemm.hip", "qmm_diag.hip", "qmm_moments.hip", "qmm_dequantize.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src, force):
    obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    deps = [path, os.path.join(CSRC, "qmm_device.h"), os.path.join(ROOT, "include", "qmm.h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    subprocess.run([HIPCC, *FLAGS, "-c", path, "-o", obj], check=True)
    return obj


def build(force=False):
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=5) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


def check_asm():
    """Compile qmm_gemm.hip to gfx950 assembly and check what the compiler cannot know about the inline-assembly
    matrix instructions and copies: (1) no accumulator register is written by v_accvgpr_write within six
    instructions in front of an MFMA that uses it (wait states), (2) every LDS copy has its base address in scalar
    registers, (3) no MFMA goes through v_accvgpr_mov copies inside the loops (at most one initialisation pass), (4) the
    kernels on the throughput path use no scratch memory, (5) the streaming kernel initialises no accumulator by a
    separate instruction and has no load the compiler knows of (outside the inline-assembly statements) behind its first MFMA (with stores outstanding the
    compiler waits for such a load with vmcnt(0), i.e. for every store), (6) the registers its inline-assembly loads fill without waiting (a tile's step
    sizes) are touched by nothing before two step barriers have passed.  Returns a list of findings (empty = clean)."""
    os.makedirs(OBJDIR, exist_ok=True)
    asm = os.path.join(OBJDIR, "qmm_gemm.s")
    subprocess.run([HIPCC, *[f for f in FLAGS if f != "-fPIC"], "--cuda-device-only", "-S",
                    os.path.join(CSRC, "qmm_gemm.hip"), "-o", asm], check=True)
    text = open(asm).read()
    findings = []
    names = list(dict.fromkeys(re.findall(r"^(_ZN3qmm\S*(?:gemm_kernel|gemm_shortk_kernel|gemm_stream_kernel)\S*):", text, flags=re.M)))
    for nm in names:
        start = text.index("\n" + nm + ":")
        end = text.index(".Lfunc_end", start)
        body = text[start:end]
        instrs = [l.strip() for l in body.split("\n")
                  if l.strip() and not l.strip().startswith((";", ".")) and not l.strip().endswith(":")]
        for k, l in enumerate(instrs):
            m = re.match(r"v_mfma\S+ a\[(\d+):(\d+)\]", l)
            if not m:
                continue
            lo, hi = int(m.group(1)), int(m.group(2))
            for q in instrs[max(0, k - 6):k]:
                w = re.match(r"v_accvgpr_write_b32 a(\d+),", q)
                if w and lo <= int(w.group(1)) <= hi:
                    findings.append(f"{nm}: v_accvgpr_write a{w.group(1)} within six instructions of '{l[:60]}'")
        for off, base in re.findall(r"global_load_lds_dwordx4 (\S+) (\S+)", body):
            if not base.startswith("s["):
                findings.append(f"{nm}: LDS copy with a vector base address ({off} {base})")
        if "gemm_stream_kernel" in nm:
            # instructions the compiler placed itself, i.e. outside the inline-assembly statements, behind the first MFMA
            own, in_asm, seen_mfma = [], False, False
            for l in (x.strip() for x in body.split("\n")):
                if "#ASMSTART" in l: in_asm = True
                elif "#ASMEND" in l: in_asm = False
                elif l.startswith("v_mfma"): seen_mfma = True
                elif seen_mfma and not in_asm and l and not l.startswith((";", ".")): own.append(l)
            late = [l for l in own if re.match(r"(global|flat|buffer|scratch)_load_(?!lds)", l)]
            if late:
                findings.append(f"{nm}: {len(late)} loads behind the first MFMA, e.g. '{late[0][:60]}'")
            if body.count("v_accvgpr_write") or body.count("v_accvgpr_mov"):
                findings.append(f"{nm}: accumulators written or moved by separate instructions")
            # the step sizes requested behind a tile's first step are waited for by nobody: the next instruction that
            # touches such a register (a copy the compiler made would be one) has to lie behind two step barriers
            first_mfma = next(k for k, l in enumerate(instrs) if l.startswith("v_mfma"))
            for k in range(first_mfma, len(instrs)):
                m = re.match(r"global_load_dword v(\d+),", instrs[k])
                if not m:
                    continue
                dst = int(m.group(1))
                for d, q in enumerate(instrs[k + 1:]):
                    if re.search(rf"\bv{dst}\b", q) or any(int(a) <= dst <= int(b) for a, b in re.findall(r"v\[(\d+):(\d+)\]", q)):
                        if sum(1 for x in instrs[k + 1:k + 1 + d] if x.startswith("s_barrier")) < 2:
                            findings.append(f"{nm}: v{dst}, loaded without a wait, is touched too early by '{q[:60]}'")
                        break
        n_acc = 128 if ("ELi4ELi1ELi4E" in nm or "shortk" in nm) else 64
        if body.count("v_accvgpr_mov") > n_acc:
            findings.append(f"{nm}: {body.count('v_accvgpr_mov')} v_accvgpr_mov (accumulators copied around MFMAs)")
        tail = text[end:end + 8000]
        sc = re.search(r"; ScratchSize: (\d+)", tail)
        targs = re.search(r"gemm_kernelI((?:Li\d+E)+)E", nm)
        fuse = int(re.findall(r"Li(\d+)E", targs.group(1))[6]) if targs else 0      # <KIND, FA, FB, TM, TG, NWN, FUSE, NSR>
        if sc and int(sc.group(1)) > 0 and targs and fuse == 0:                       # codes-in kernels: the throughput path
            findings.append(f"{nm}: {sc.group(1)} bytes of scratch per lane")
        if sc and int(sc.group(1)) > 0 and ("shortk" in nm or "gemm_stream_kernel" in nm):
            findings.append(f"{nm}: {sc.group(1)} bytes of scratch per lane")
    return names, findings


if __name__ == "__main__":
    if "--check-asm" in sys.argv:
        kernels, found = check_asm()
        print(f"{len(kernels)} kernels scanned")
        for f in found:
            print("FINDING:", f)
        sys.exit(1 if found else 0)
    print(build(force="--force" in sys.argv))
