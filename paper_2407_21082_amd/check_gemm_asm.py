"""Static check of the batched kernel's hand-counted loads in the compiled gfx950 assembly.

`csrc/eh_gemm.hip` loads activation fragments with `global_load_dwordx4` instructions the
compiler does not track (inline asm), and waits for them with `s_waitcnt vmcnt(N)` on a
compile-time count of younger loads.  That is only sound if, in the generated code,

  * no instruction reads or writes a destination register of such a load while the load
    may still be in flight (a register handed out again too early lets the returning data
    overwrite an address or an operand), and
  * no path reaches the end of the program with such a load still in flight.

This module proves both properties on the assembly text: for every `global_load_dwordx4`
into VGPRs (and every `ds_read_b128`) that comes from an inline-asm statement it walks every path of the kernel's control-flow graph forward from the load,
counting vector-memory loads issued after it (loads return in order, so
`s_waitcnt vmcnt(N)` guarantees the load has landed once at least N younger ones were
issued), and reports any instruction that names one of the load's destination registers
before such a wait.  The build runs it on every `gemm_stats_kernel` instantiation and
fails on a finding, so a compiler or source change cannot silently bring the hazard back.

    python -m paper_2407_21082_amd.check_gemm_asm file.s
"""
from __future__ import annotations

import re
import sys
from collections import deque

KERNEL_RE = re.compile(r"^(_Z\w*gemm(?:32)?_(?:stats|kl)_kernel\w*):")
LABEL_RE = re.compile(r"^(\.L\w+):")
VREG_RE = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
UNTRACKED_RE = re.compile(r"^global_load_dwordx4\s+v\[(\d+):(\d+)\]\s*,")  # any addressing form
VMCNT_RE = re.compile(r"vmcnt\((\d+)\)")
VMEM_RE = re.compile(r"^(global_|buffer_|flat_|scratch_)")
# only loads are counted as "younger": a store may retire ahead of an older load
VLOAD_RE = re.compile(r"^(global|buffer|flat|scratch)_load")
LONG_BRANCH_RE = re.compile(r"\((\.L\w+)-\.Lpost_getpc\d+\)")


def _vregs(text: str) -> set:
    regs = set()
    for m in VREG_RE.finditer(text):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


def split_kernels(asm: str) -> dict:
    """name -> list of lines of each gemm_stats_kernel body."""
    out, name, body = {}, None, []
    for line in asm.split("\n"):
        m = KERNEL_RE.match(line)
        if m:
            name, body = m.group(1), []
            continue
        if name is not None:
            if line.startswith(".Lfunc_end"):
                out[name] = body
                name = None
            else:
                body.append(line)
    return out


class Program:
    def __init__(self, lines):
        self.ins = []        # instruction text (mnemonic + operands, comments stripped)
        self.note = []       # the comment that followed it on its line ("" if none)
        self.by_hand = []    # the instruction comes from an inline-asm statement of the source
        self.label_at = {}   # label -> index of the next instruction
        in_asm = False
        for line in lines:
            m = LABEL_RE.match(line)
            if m:
                self.label_at[m.group(1)] = len(self.ins)
                continue
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            t, _, note = line.partition(";")
            t = t.strip()
            if not t or t.startswith("."):
                continue
            self.ins.append(t)
            self.note.append(note.strip())
            self.by_hand.append(in_asm)
        n = len(self.ins)
        self.succ = [None] * n
        for i, t in enumerate(self.ins):
            op = t.split()[0]
            if op == "s_endpgm":
                self.succ[i] = ()
            elif op == "s_branch":
                self.succ[i] = (self.label_at[t.split()[1]],)
            elif op.startswith("s_cbranch"):
                self.succ[i] = (self.label_at[t.split()[1]], i + 1)
            elif op.startswith("s_setpc"):
                # branch relaxation: s_getpc / s_add_u32 (.Ltarget-.Lpost_getpc) / s_addc / s_setpc
                tgt = None
                for j in range(i - 1, max(i - 6, -1), -1):
                    m = LONG_BRANCH_RE.search(self.ins[j])
                    if m:
                        tgt = self.label_at[m.group(1)]
                        break
                if tgt is None:
                    raise ValueError("indirect branch with unknown target: " + t)
                self.succ[i] = (tgt,)
            else:
                self.succ[i] = (i + 1,) if i + 1 < n else ()


class LoadClass:
    """A kind of load whose completion is awaited through one `s_waitcnt` counter."""

    def __init__(self, what, load_re, younger_re, wait_re, disorder_re=None):
        self.what = what
        self.load_re = re.compile(load_re)        # groups: first and last destination VGPR
        self.younger_re = re.compile(younger_re)  # instructions that return in order behind it
        self.wait_re = re.compile(wait_re)        # the counter field of s_waitcnt
        # instructions on the same counter that may return out of order with the load:
        # once one is in flight only a wait for zero proves the load has landed
        self.disorder_re = re.compile(disorder_re) if disorder_re else None


VM_LOADS = LoadClass("global load", r"^global_load_dwordx4\s+v\[(\d+):(\d+)\]\s*,",
                     r"^(global|buffer|flat|scratch)_load", r"vmcnt\((\d+)\)")
LDS_LOADS = LoadClass("LDS read", r"^ds_read_b128\s+v\[(\d+):(\d+)\]\s*,", r"^ds_",
                      r"lgkmcnt\((\d+)\)", r"^s_(load|buffer_load|scratch_load|sendmsg|memtime|memrealtime)")


def check_kernel(lines, max_report=5, classes=(VM_LOADS, LDS_LOADS)):
    """Findings (strings) and number of loads examined for one kernel body."""
    prog = Program(lines)
    ins = prog.ins
    regs_of = [_vregs(t) for t in ins]
    findings = []
    n_loads = 0
    for cls in classes:
        is_younger = [bool(cls.younger_re.match(t)) for t in ins]
        disorders = [bool(cls.disorder_re and cls.disorder_re.match(t)) for t in ins]
        wait_n = []
        for t in ins:
            m = cls.wait_re.search(t) if t.startswith("s_waitcnt") else None
            wait_n.append(int(m.group(1)) if m else None)
        for i, t in enumerate(ins):
            m = cls.load_re.match(t)
            # loads the compiler emitted itself are tracked by its own wait counts (it may even
            # reuse a destination whose value is dead: loads return in order); the hand-counted
            # ones are those of the source's inline-asm statements
            if not m or not prog.by_hand[i]:
                continue
            n_loads += 1
            dest = set(range(int(m.group(1)), int(m.group(2)) + 1))
            seen = set()
            todo = deque((s, 0, False) for s in prog.succ[i])
            while todo:
                pc, younger, mixed = todo.popleft()
                if (pc, younger, mixed) in seen:
                    continue
                seen.add((pc, younger, mixed))
                if wait_n[pc] is not None and (wait_n[pc] == 0 or (not mixed and younger >= wait_n[pc])):
                    continue                      # landed on this path
                if regs_of[pc] & dest:
                    findings.append(f"{cls.what} #{i} `{t}`: `{ins[pc]}` (#{pc}) touches its destination "
                                    f"with only {younger} younger loads and no wait")
                    break
                if ins[pc].startswith("s_endpgm"):
                    findings.append(f"{cls.what} #{i} `{t}` still in flight at s_endpgm (#{pc})")
                    break
                y2 = min(younger + 1, 64) if is_younger[pc] else younger
                for s in prog.succ[pc]:
                    todo.append((s, y2, mixed or disorders[pc]))
            if len(findings) >= max_report:
                return findings, n_loads
    return findings, n_loads


STEP_SYNC_RE = re.compile(r"^s_waitcnt vmcnt\((\d+)\)(?: lgkmcnt\(0\))?$")


def check_step_counts(name, lines, max_report=5):
    """The waits count on every k-step issuing the same loads.  A step sync is a
    `s_waitcnt vmcnt(N)` with N > 0 that the kernel source marks with the comment
    `; step-sync` (the compiler's own waits are not step syncs).  On every control-flow path from one step sync to the next, the loads
    issued (DMA + register loads) must divide the next sync's N -- by the same factor (the
    k-steps a load may stay in flight beyond the next one) everywhere in the kernel -- and
    nothing else may use vector memory.  Paths end at a pass boundary (`vmcnt(0)`)."""
    prog = Program(lines)
    ins = prog.ins
    sync_n = {}
    for i, t in enumerate(ins):
        m = STEP_SYNC_RE.match(t)
        if m and int(m.group(1)) > 0 and "step-sync" in prog.note[i]:
            sync_n[i] = int(m.group(1))
    findings, depths, checked = [], set(), 0
    for start in sync_n:
        seen = set()
        todo = [(s, 0, 0) for s in prog.succ[start]]
        while todo and len(findings) < max_report:
            pc, dma, reg = todo.pop()
            if (pc, dma, reg) in seen or dma + reg > 64:
                continue
            seen.add((pc, dma, reg))
            t = ins[pc]
            if pc in sync_n:
                if dma + reg == 0:
                    pass                  # prologue: operands of step 0 come from LDS only
                else:
                    checked += 1
                    n = sync_n[pc]
                    if dma == 0 or reg == 0 or n % (dma + reg) != 0:
                        findings.append(f"k-step from sync #{start} to sync #{pc}: {dma} DMA + {reg} register "
                                        f"loads, wait vmcnt({n}) (want a multiple of the loads)")
                    else:
                        depths.add(n // (dma + reg))
                    continue
            if t.startswith("s_endpgm") or (t.startswith("s_waitcnt") and "vmcnt(0)" in t):
                continue                  # pass boundary
            if t.startswith("global_load_lds_dwordx4"):
                dma += 1
            elif UNTRACKED_RE.match(t):
                reg += 1
            elif VMEM_RE.match(t):
                findings.append(f"k-step after sync #{start}: other vector memory `{t}` (#{pc})")
                continue
            for s in prog.succ[pc]:
                todo.append((s, dma, reg))
    if len(depths) > 1:
        findings.append(f"k-steps wait with different depths: {sorted(depths)}")
    if checked == 0:
        findings.append("no k-step found between step syncs")
    return findings, checked


def check_asm(asm: str):
    """(findings, kernels checked, loads checked) for every gemm_stats_kernel in the text."""
    kernels = split_kernels(asm)
    findings, loads = [], 0
    for name, body in kernels.items():
        f, n = check_kernel(body)
        g, _ = check_step_counts(name, body)
        loads += n
        findings += [f"{name}: {x}" for x in f + g]
    return findings, len(kernels), loads


def main(argv):
    if len(argv) != 2:
        print(__doc__)
        return 2
    findings, nk, nl = check_asm(open(argv[1]).read())
    for f in findings:
        print("HAZARD", f)
    print(f"check_gemm_asm: {nk} kernels, {nl} untracked loads, {len(findings)} findings")
    return 1 if findings or nk == 0 else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
