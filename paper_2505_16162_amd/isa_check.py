"""Static checks of the compiled ISA of the kernels that place their own loads.

The draft GEMV and the verification GEMM issue their global loads from inline assembly and wait for them
with their own `s_waitcnt vmcnt(N)` (see `stream_load` / `stream_wait` in csrc/kernels_bf16.h). The compiler
does not know that such a register is still being written by the memory system, so two things it may do
are fatal and silent: spilling such a register, and copying it (a `v_mov` that joins two register
assignments of the same variable) before the wait. The first is caught from the compiler's resource
remarks (build.py); this module catches the second from the assembly text:

* `inflight_flags`  a forward dataflow over the kernel's control-flow graph. State: for every vector
  register that is the target of a hand-placed load, the least number of younger hand-placed loads issued
  since, over all paths; a hand-placed `vmcnt(N)` retires the registers with at least N younger loads. Any
  other instruction that touches a register still in the state is flagged. Exact for kernels whose loops
  have no correlated branches (the GEMV: zero flags required).
* `weight_register_copies`  for kernels where that analysis sees infeasible paths (the verification GEMM:
  chunk and round conditions are correlated): every `v_mov` / `v_accvgpr` / `scratch` instruction between
  the first streaming load and the last hand-placed wait that READS a register of the weight stream.
  Those registers are read by nothing but the matrix instructions there, so any hit is a copy or a spill.
"""
import re

_LABEL = re.compile(r"^(\.LBB\d+_\d+):")


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def kernel_bodies(asm_text, name_fragment):
    """[(mangled name, [lines])] of every kernel whose mangled name contains the fragment."""
    lines = asm_text.split("\n")
    out = []
    i = 0
    while i < len(lines):
        ln = lines[i]
        if ln.startswith("_Z") and ":" in ln and name_fragment in ln.split(":")[0]:
            name = ln.split(":")[0]
            j = i + 1
            while j < len(lines) and not lines[j].startswith(".Lfunc_end"):
                j += 1
            out.append((name, lines[i + 1:j]))
            i = j
        i += 1
    return out


def _instructions(body):
    """(line number, text, inside an inline-asm block) of every instruction; labels as (n, 'LABEL name', False)."""
    in_asm = False
    for n, raw in enumerate(body):
        t = raw.strip()
        m = _LABEL.match(t)
        if m:
            yield n, "LABEL " + m.group(1), False
            continue
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t.startswith((";", ".")):
            continue
        t = t.split(";")[0].strip()
        if t:
            yield n, t, in_asm


def inflight_flags(body):
    """List of (line, instruction, register, reason); empty when no instruction can touch a register whose
    hand-placed load has not been retired by a hand-placed wait."""
    blocks, cur = [], {"label": "_entry", "ins": []}
    for n, t, ia in _instructions(body):
        if t.startswith("LABEL "):
            blocks.append(cur)
            cur = {"label": t[6:], "ins": []}
            continue
        cur["ins"].append((n, t, ia))
        if t.startswith(("s_branch", "s_cbranch", "s_endpgm")):
            blocks.append(cur)
            cur = {"label": None, "ins": []}
    blocks.append(cur)
    blocks = [b for b in blocks if b["ins"] or b["label"]]
    index = {b["label"]: i for i, b in enumerate(blocks) if b["label"]}
    succ = []
    for i, b in enumerate(blocks):
        s = []
        last = b["ins"][-1][1] if b["ins"] else ""
        if last.startswith("s_endpgm"):
            pass
        elif last.startswith("s_branch"):
            s.append(index[last.split()[1]])
        else:
            if last.startswith("s_cbranch"):
                s.append(index[last.split()[1]])
            if i + 1 < len(blocks):
                s.append(i + 1)
        succ.append(s)

    def transfer(state, block, report):
        st = dict(state)
        for n, t, ia in block["ins"]:
            if ia and t.startswith("global_load"):
                dst = _regs(t.split(",")[0])
                if report is not None:
                    for r in _regs(t):
                        if r in st:
                            report.append((n, t, r, "hand-placed load names a register with a load in flight"))
                for r in st:
                    st[r] += 1
                for r in dst:
                    st[r] = 0
            elif ia and t.startswith("s_waitcnt"):
                m = re.search(r"vmcnt\((\d+)\)", t)
                if m:
                    keep = int(m.group(1))
                    st = {r: c for r, c in st.items() if c < keep}
            elif t.startswith("s_waitcnt"):
                pass        # the compiler's own waits are computed without knowledge of the hand-placed loads
            elif report is not None:
                for r in _regs(t):
                    if r in st:
                        report.append((n, t, r, "load in flight (%d younger loads at least)" % st[r]))
        return st

    state_in = [None] * len(blocks)
    state_in[0] = {}
    work = [0]
    while work:
        i = work.pop()
        out = transfer(state_in[i], blocks[i], None)
        for j in succ[i]:
            if state_in[j] is None:
                new = dict(out)
            else:
                new = dict(state_in[j])
                for r, c in out.items():
                    new[r] = min(new.get(r, c), c)
            if new != state_in[j]:
                state_in[j] = new
                work.append(j)
    report = []
    for i, b in enumerate(blocks):
        if state_in[i] is not None:
            transfer(state_in[i], b, report)
    seen, flags = set(), []
    for n, t, r, why in report:
        if n not in seen:
            seen.add(n)
            flags.append((n, t, r, why))
    return flags


def weight_register_copies(body):
    """List of (line, instruction): register copies and spills that read a register of the weight stream (the
    targets of the nontemporal hand-placed loads) between the first such load and the last hand-placed wait."""
    ins = list(_instructions(body))
    weight, first, last_wait = set(), None, None
    for n, t, ia in ins:
        if ia and t.startswith("global_load") and t.rstrip().endswith(" nt"):
            weight |= _regs(t.split(",")[0])
            if first is None:
                first = n
        if ia and t.startswith("s_waitcnt"):
            last_wait = n
    if first is None:
        return []
    hits = []
    for n, t, ia in ins:
        if ia or not (first < n < last_wait):
            continue
        # the registers an instruction READS: everything behind the first comma (a store has no destination)
        if t.startswith(("v_mov", "v_accvgpr")):
            read = _regs(t.split(",", 1)[1]) if "," in t else set()
        elif t.startswith("scratch_store"):
            read = _regs(t)
        else:
            continue
        if read & weight:
            hits.append((n, t))
    return hits
