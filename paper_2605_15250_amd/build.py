"""Builds libgqla.so (the C-ABI library, gfx950 code objects) in-tree with hipcc, and the oracle's C parts if any."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgqla.so")

SOURCES = ["gqla_api.hip", "gqla_f32.hip", "gqla_gqa_bf16.hip", "gqla_absorb_bf16.hip", "gqla_gemm_bf16.hip",
           "gqla_probe.hip", "gqla_fp8.hip", "gqla_step_ops.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str, extra) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


# Kernels listed here keep data in accumulation registers behind the compiler's back: the absorb decode addresses
# them by name in inline assembly (the compiler knows them only as clobbered, so it must never park values of its own
# there), the expansion loads them asynchronously from inline assembly (a compiler-made copy before the wait would copy
# stale data).  The compiler touches accumulation registers itself (v_accvgpr_write / _read / _mov outside the assembly
# blocks) only when it runs out of ordinary registers: the build checks the generated assembly and refuses such a
# kernel instead of shipping silent corruption.
NAMED_AGPR_SOURCES = {"gqla_absorb_bf16.hip": ["decode_absorb_bf16_kernel", "decode_absorb_shared_bf16_kernel", "decode_absorb_fp8_kernel"],
                      "gqla_gemm_bf16.hip": ["expand_bf16_kernel"]}


# Kernels that fetch page-table entries with a scalar load written in inline assembly and wait for it by hand much
# later: a compiler-made copy of that register ahead of the wait would read it while the load is pending (the compiler
# cannot see the load, so nothing protects such a read).  The build scans the generated assembly for any read of the
# register between the load and the next wait for scalar memory and refuses the kernel.
HAND_SCALAR_LOAD_KERNELS = {"gqla_absorb_bf16.hip": ["decode_absorb_bf16_kernel", "decode_absorb_shared_bf16_kernel"],
                            "gqla_gqa_bf16.hip": ["decode_gqa_bf16_kernel"]}


# Kernels whose loops wait on hand-counted numbers of outstanding vector-memory instructions (s_waitcnt vmcnt(N) written
# for the loads the source issues): a register spill would add scratch loads and stores of the compiler's own to that
# count and silently break the waits.  The build reads the compiler's resource report and refuses any vector-register
# spill or scratch use in them.
COUNTED_WAIT_KERNELS = {"gqla_absorb_bf16.hip": ["decode_absorb_bf16_kernel", "decode_absorb_shared_bf16_kernel"],
                        "gqla_gemm_bf16.hip": ["expand_bf16_kernel"],
                        "gqla_gqa_bf16.hip": ["decode_gqa_bf16_kernel"],
                        "gqla_step_ops.hip": ["out_proj_bf16_kernel"]}


def _reads_register(instr: str, reg: str) -> bool:
    """Does this instruction read scalar register `reg`?  The first operand is the destination, except for compares,
    branches and stores, which only read."""
    parts = instr.split(None, 1)
    if len(parts) < 2:
        return False
    ops = [o.strip() for o in parts[1].split(",")]
    if not parts[0].startswith(("s_cmp", "s_bitcmp", "v_cmp", "s_cbranch", "global_store", "ds_write", "buffer_store", "s_store")):
        ops = ops[1:]
    num = int(reg[1:])
    for o in ops:
        if re.fullmatch(r"%s" % reg, o):
            return True
        m = re.fullmatch(r"s\[(\d+):(\d+)\]", o)     # a register range that contains it
        if m and int(m.group(1)) <= num <= int(m.group(2)):
            return True
    return False


def _check_device_code(src: str, extra) -> None:
    """One device-only compile to assembly with the resource report: no compiler-made accumulation-register traffic in
    the kernels of NAMED_AGPR_SOURCES, no spills and no scratch in those of COUNTED_WAIT_KERNELS."""
    asm_path = os.path.join(BUILD, os.path.splitext(src)[0] + ".s")
    cmd = [_hipcc(), *FLAGS, *extra, "--cuda-device-only", "-S", "-Rpass-analysis=kernel-resource-usage",
           os.path.join(CSRC, src), "-o", asm_path]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for %s:\n%s" % (src, r.stderr))
    agpr_kernels = NAMED_AGPR_SOURCES.get(src, [])
    sload_kernels = HAND_SCALAR_LOAD_KERNELS.get(src, [])
    kernels = sorted(set(agpr_kernels) | set(sload_kernels))
    current, in_asm, seen_labels = None, False, set()
    pending = None   # scalar register that a hand-written s_load_dword has in flight (until the hand-written wait)
    with open(asm_path) as fh:
        for line in fh:
            t = line.strip()
            m = re.match(r"^([A-Za-z_$][\w$.]*):", line)      # a function label ("name:" at the start of the line, maybe a comment behind)
            if m:
                current = next((k for k in kernels if k in m.group(1)), None)
                seen_labels.add(current)
                pending = None
            elif t.startswith(".Lfunc_end"):
                current = pending = None
            elif ";;#ASMSTART" in t:
                in_asm = True
            elif ";;#ASMEND" in t:
                in_asm = False
            elif current in agpr_kernels and not in_asm and t.startswith("v_accvgpr_"):
                raise RuntimeError("%s: the compiler uses accumulation registers of its own in %s (%s); "
                                   "lower the kernel's VGPR pressure" % (src, current, t))
            elif current in sload_kernels and in_asm and t.startswith("s_load_dword "):
                pending = t.split()[1].rstrip(",")
            elif current and pending and t.startswith("s_waitcnt") and "lgkmcnt(0)" in t:   # hand-written or the compiler's
                pending = None
            elif current and pending and not in_asm and not t.startswith((";", ".")) and _reads_register(t, pending):
                # (in the order of the listing, which is the order of execution on the paths where this can happen:
                # the load and its wait sit in one loop body; a write to the register belongs to the branch that
                # computes the value without a load)
                raise RuntimeError("%s: %s reads %s while the scalar load issued by hand is still in flight (%s): the "
                                   "compiler cannot see that load, so no wait protects this read" % (src, current, pending, t))
    missing = [k for k in kernels if k not in seen_labels]
    if missing:
        raise RuntimeError("%s: no function label found for %s (kernel renamed?)" % (src, ", ".join(missing)))
    # resource report: "remark: Function Name: <mangled>" followed by one remark per figure
    watched = COUNTED_WAIT_KERNELS.get(src, [])
    current, seen = None, set()
    for line in r.stderr.splitlines():
        if "remark:" not in line:
            continue
        body = line.split("remark:", 1)[1].strip()
        if body.startswith("Function Name:"):
            current = next((k for k in watched if k in body), None)
            if current:
                seen.add(current)
            continue
        if not current:
            continue
        # (scalar registers spilled into lanes of a vector register cost no memory instruction and are allowed)
        for key in ("ScratchSize [bytes/lane]:", "VGPRs Spill:"):
            if body.startswith(key):
                val = body[len(key):].split("[")[0].strip()
                if val != "0":
                    raise RuntimeError("%s: %s has %s %s; its hand-counted memory waits need a spill-free kernel"
                                       % (src, current, key, val))
    missing = [k for k in watched if k not in seen]
    if missing:
        raise RuntimeError("%s: no resource report for %s (kernel renamed?)" % (src, ", ".join(missing)))


def build(extra_flags=(), jobs: int = 5) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        checks = [ex.submit(_check_device_code, src, list(extra_flags))
                  for src in sorted(set(NAMED_AGPR_SOURCES) | set(COUNTED_WAIT_KERNELS))]
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
        for c in checks:
            c.result()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


HOSTCHECK_LIB = os.path.join(BUILD, "hostcheck", "libgqla_hostcheck.so")
HOST_SANITIZERS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                   "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-g", "-Xarch_host", "-O1"]


def build_hostcheck(jobs: int = 8):
    """The same library with its HOST code instrumented by the address and undefined-behaviour sanitizers (the GPU code
    objects are built as usual and are not instrumented): what the CPU tests load to run the planner, the argument
    validation and the left-inverse solve under the sanitizers.  Returns (library, sanitizer runtime to preload into an
    uninstrumented interpreter)."""
    out = os.path.join(BUILD, "hostcheck")
    os.makedirs(out, exist_ok=True)

    def one(src):
        obj = os.path.join(out, os.path.splitext(src)[0] + ".o")
        r = subprocess.run([_hipcc(), *FLAGS, *HOST_SANITIZERS, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc (host sanitizers) failed for %s:\n%s" % (src, r.stderr))
        return obj
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, SOURCES))
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address",
                        "-fsanitize=undefined", "-shared-libsan", "-Wno-option-ignored", "-o", HOSTCHECK_LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link (host sanitizers) failed:\n" + r.stderr)
    rt = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        raise RuntimeError("address-sanitizer runtime not found next to the compiler: %r" % rt)
    return HOSTCHECK_LIB, rt


if __name__ == "__main__":
    print(build(sys.argv[1:]))
