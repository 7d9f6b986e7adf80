"""Compile the HIP library for gfx950 into paper_2604_26666_amd/libfact_gemm.so.

One translation unit per tile configuration (csrc/configs.def), compiled in parallel,
plus the auxiliary kernels and the C ABI.  hipcc cross-compiles without a GPU.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfact_gemm.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-I", CSRC]


def configs():
    rows = []
    with open(os.path.join(CSRC, "configs.def")) as f:
        for line in f:
            m = re.match(r"\s*FACT_CFG\(\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*\)", line)
            if m:
                rows.append(tuple(int(x) for x in m.groups()))
    return rows


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def resource_usage(text):
    """Parse the compiler's kernel-resource-usage remarks: {kernel: {field: int}}."""
    res, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = res.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z /\[\]]+): (\d+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return res


_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+))")


def _regs(operand):
    """Set of ('v'|'a', index) named by one assembly operand."""
    out = set()
    for m in _REG.finditer(operand):
        kind = m.group(1)
        if m.group(4) is not None:
            out.add((kind, int(m.group(4))))
        else:
            out.update((kind, i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def check_asm_mfma_hazards(asm_text, kernel_filter="attn_fwd_kernel"):
    """The GEMM and attention kernels issue their MFMAs through inline asm, so the compiler keeps none of the
    wait states the matrix pipe needs around them.  Two cases are checked in the generated code:
    a vector-ALU instruction writing a register that one of the next two instructions, an asm
    MFMA, reads as an operand (seen on the GPU: the MFMA used the register's old contents); and a
    vector-ALU instruction reading an MFMA's result with fewer than 5 instructions or 20 s_nop
    cycles in between.  Returns a list of findings (empty = fine)."""
    findings = []
    checked = 0
    for m in re.finditer(r"^(_Z\w+):[^\n]*\n(.*?)^\s*s_endpgm", asm_text, re.S | re.M):
        name, kern = m.group(1), m.group(2)
        if kernel_filter not in name:
            continue
        checked += 1
        insts = []                      # (text, is_asm_mfma, valu_dest_regs, src_regs)
        in_asm = False
        for line in kern.splitlines():
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if t.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if not t or t.startswith((";", ".", "//")) or t.endswith(":"):
                continue
            op, _, rest = t.partition(" ")
            ops = [o.strip() for o in rest.split(",")]
            is_mfma = op.startswith("v_mfma")
            dest = _regs(ops[0]) if ops and op.startswith("v_") else set()
            srcs = set().union(*[_regs(o) for o in ops[1:]]) if len(ops) > 1 else set()
            nop_cycles = int(ops[0]) + 1 if op == "s_nop" and ops and ops[0].isdigit() else 0
            insts.append((t, is_mfma and in_asm, dest, srcs, op, nop_cycles))
        for i, (t, asm_mfma, dest, srcs, op, _) in enumerate(insts):
            if asm_mfma:
                for k in (1, 2):
                    if i - k >= 0:
                        pt, p_mfma, pdest, _, pop, _ = insts[i - k]
                        if pop.startswith("v_") and not pop.startswith("v_mfma") and pdest & srcs:
                            findings.append(f"{name}: '{pt}' writes an operand of '{t}' {k} instruction(s) before it")
            elif op.startswith("v_") and not op.startswith("v_mfma"):
                need = srcs | dest
                cycles = 0
                for k in range(1, 6):
                    if i - k < 0:
                        break
                    pt, p_mfma, pdest, _, pop, pn = insts[i - k]
                    if cycles >= 20:
                        break
                    if p_mfma and pdest & need:
                        findings.append(f"{name}: '{t}' touches the result of '{pt}' {k} instruction(s) after it")
                    cycles += pn
    if checked == 0:
        findings.append("no kernel matching '" + kernel_filter + "' found in the generated code: nothing was checked")
    return findings


def check_accumulators_untouched(asm_text, kernel_filter="gemm_kernel"):
    """The GEMM kernel keeps its accumulators in accumulation registers that only its inline assembly
    names (declared as written by every statement that writes them).  Any instruction the compiler
    emits by itself that names an accumulation register there - a copy, a spill into that register
    file - could overwrite a tile: refuse such a build."""
    findings = []
    for m in re.finditer(r"^(_Z\w+):[^\n]*\n(.*?)^\s*s_endpgm", asm_text, re.S | re.M):
        name, kern = m.group(1), m.group(2)
        if kernel_filter not in name:
            continue
        in_asm = False
        for line in kern.splitlines():
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if t.startswith(";;#ASMEND"):
                in_asm = False
                continue
            if in_asm or not t or t.startswith((";", ".", "//")) or t.endswith(":"):
                continue
            if re.search(r"\ba(\d+|\[\d+:\d+\])", t.partition(" ")[2]) or t.startswith("v_accvgpr"):
                findings.append(f"{name}: the compiler emitted '{t}', which names an accumulation register")
                if len(findings) > 20:
                    return findings
    return findings


def check_wide_store_hazards(asm_text):
    """A buffer store of more than 64 bits whose data registers are overwritten by the vector ALU in the
    very next instruction needs one wait state (the ISA manual's table of manually inserted wait
    states: "VMEM store of more than 64 bits, then a VALU write of the store's data registers").  The
    compiler's hazard pass applies the rule only to stores whose scalar-offset operand is a constant;
    on gfx950 a store with a register there was seen to pick up the overwriting value in some lanes.
    The sources therefore keep that operand constant; this scan refuses a build in which a wide
    buffer store with a register offset is followed directly by a write to its data."""
    findings = []
    insts = []
    for line in asm_text.splitlines():
        t = line.strip()
        if not t or t.startswith((";", ".", "//")) or t.endswith(":"):
            continue
        insts.append(t)
    for i, t in enumerate(insts[:-1]):
        op, _, rest = t.partition(" ")
        if not (op.startswith("buffer_store_dwordx4") or op.startswith("buffer_store_dwordx3")):
            continue
        ops = [o.strip() for o in rest.split(",")]
        if len(ops) < 4:
            continue
        soffset = ops[3].split()[0]
        if not re.match(r"^(s\d+|m0|vcc_lo|vcc_hi|ttmp\d+)$", soffset):
            continue                                  # constant (or off): the compiler keeps the wait state itself
        data = _regs(ops[0])
        nxt = insts[i + 1]
        nop, _, nrest = nxt.partition(" ")
        if nop.startswith("v_") and data & _regs(nrest.split(",")[0]):
            findings.append(f"'{nxt}' overwrites the data of '{t}' in the next cycle")
    return findings


def write_acc_regs(path=os.path.join(CSRC, "acc_regs.inc")):
    """csrc/acc_regs.inc: one line per accumulator tile, naming its four accumulation registers (the kernel
    addresses them by name in its inline assembly; register names cannot be computed by templates)."""
    text = ("// GENERATED by paper_2604_26666_amd/build.py (write_acc_regs): accumulator tile T lives in the accumulation\n"
            "// registers a[4T .. 4T+3].  FACT_ACC_TILE(T, first, second, third, last register).\n" +
            "".join(f"FACT_ACC_TILE({t}, {4 * t}, {4 * t + 1}, {4 * t + 2}, {4 * t + 3})\n" for t in range(64)))
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
    return path


def build(jobs=None, verbose=False, extra_flags=(), lib=LIB, obj_dir=OBJ):
    """extra_flags / lib / obj_dir exist for experiments (a variant library beside the product one)."""
    write_acc_regs()
    OBJ = obj_dir
    LIB = lib
    FLAGS = list(globals()["FLAGS"]) + list(extra_flags)
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    units = []
    for (cid, bm, bn, wm, wn, bk, st) in configs():
        obj = os.path.join(OBJ, f"inst{cid}.o")
        units.append((obj, [HIPCC] + FLAGS + ["-Rpass-analysis=kernel-resource-usage", f"-DFACT_ID={cid}", f"-DFACT_BM={bm}", f"-DFACT_BN={bn}",
                                              f"-DFACT_WM={wm}", f"-DFACT_WN={wn}", f"-DFACT_BK={bk}", f"-DFACT_STAGES={st}",
                                              "-c", os.path.join(CSRC, "inst.hip"), "-o", obj]))
    for name in ("aux_kernels", "fact_api", "attention", "block"):
        obj = os.path.join(OBJ, name + ".o")
        units.append((obj, [HIPCC] + FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, name + ".hip"), "-o", obj]))
    # the same kernels once more as assembly text, for the check of the inline-asm MFMAs below
    asm_units = []
    for (cid, bm, bn, wm, wn, bk, st) in configs():
        asm_units.append((os.path.join(OBJ, f"inst{cid}.s"), "gemm_kernel",
                          [HIPCC] + FLAGS + [f"-DFACT_ID={cid}", f"-DFACT_BM={bm}", f"-DFACT_BN={bn}", f"-DFACT_WM={wm}", f"-DFACT_WN={wn}",
                                             f"-DFACT_BK={bk}", f"-DFACT_STAGES={st}", "--cuda-device-only", "-S",
                                             os.path.join(CSRC, "inst.hip"), "-o", os.path.join(OBJ, f"inst{cid}.s")]))
    asm_units.append((os.path.join(OBJ, "attention.s"), "attn_fwd_kernel",
                      [HIPCC] + FLAGS + ["--cuda-device-only", "-S", os.path.join(CSRC, "attention.hip"), "-o", os.path.join(OBJ, "attention.s")]))
    usage = {}
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        asm_jobs = [ex.submit(_run, u[2]) for u in asm_units]
        for out in ex.map(lambda u: _run(u[1]), units):
            usage.update(resource_usage(out))
            rest = "\n".join(l for l in out.splitlines() if "kernel-resource-usage" not in l and not re.match(r"\s*(\d+ \| |\| |In file included)", l))
            if verbose and rest.strip():
                print(rest)
    # The main kernel issues LDS reads through inline asm the compiler does not track: a spilled
    # fragment register would be stored before its data has arrived.  Refuse such a build.
        for j in asm_jobs:
            j.result()
    bad = {k: v for k, v in usage.items() if ("gemm_kernel" in k or "attn_fwd_kernel" in k)
           and (v.get("ScratchSize [bytes/lane]", 0) or v.get("VGPRs Spill", 0))}
    if verbose:
        for k, v in sorted(usage.items()):
            if "gemm_kernel" in k or "attn_fwd_kernel" in k:
                print(f"{k}: VGPRs {v.get('VGPRs')} AGPRs {v.get('AGPRs')} SGPR spills {v.get('SGPRs Spill')} scratch {v.get('ScratchSize [bytes/lane]')}")
    if bad and not os.environ.get("FACT_ALLOW_SPILLS"):
        raise RuntimeError("register spills in a kernel with untracked LDS reads (a spill could store a register before its data arrives): " +
                           "; ".join(f"{k}: {v}" for k, v in bad.items()))
    # inline-asm MFMAs (GEMM and attention kernels): check the generated code for the wait-state cases
    hazards = []
    for path, kernel, _ in asm_units:
        text = open(path).read()
        hazards += check_asm_mfma_hazards(text, kernel_filter=kernel)
        hazards += [f"{os.path.basename(path)}: {h}" for h in check_wide_store_hazards(text)]
        if kernel == "gemm_kernel":
            hazards += check_accumulators_untouched(text)
    if hazards and not os.environ.get("FACT_ALLOW_ASM_HAZARDS"):      # (override for timing experiments only)
        raise RuntimeError("wait-state hazards in the generated code:\n  " + "\n  ".join(hazards[:20]))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + [u[0] for u in units])
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
