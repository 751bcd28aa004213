"""Walk the control-flow graph of AMDGPU assembly text: for every matrix instruction, the fewest wait states on
ANY path to the first later instruction, other than a matrix instruction, that reads one of its result registers.
One instruction counts as one wait state, `s_nop N` as N + 1.  The compiler inserts the wait states the hardware
needs between a matrix instruction and a reader of its result from the paths it looks at; this walk looks at all
of them (both ways at every conditional branch), which is how a short path can be found that the compiler did not
cover."""
import re


def _regs(tok):
    out = set()
    for a, b in re.findall(r"\b[va]\[(\d+):(\d+)\]", tok):
        out |= set(range(int(a), int(b) + 1))
    for a in re.findall(r"\b[va](\d+)\b", tok):
        out.add(int(a))
    return out


def kernels(asm_text):
    """{mangled name: (instructions, {label: index})} for every function of the file."""
    out = {}
    for m in re.finditer(r"^(_Z\S+):.*$", asm_text, flags=re.M):
        end = asm_text.find(".Lfunc_end", m.end())
        ins, labels = [], {}
        for line in asm_text[m.end():end].splitlines():
            t = line.split(";")[0].strip()
            if not t:
                continue
            if re.match(r"^\.L\S+:$", t):
                labels[t[:-1]] = len(ins)
            elif not t.startswith("."):
                ins.append(t)
        out[m.group(1)] = (ins, labels)
    return out


def shortest_reads(ins, labels, opcode_prefix, limit=64):
    """[(wait states, matrix instruction, reader)] for the shortest path from each matrix instruction whose
    mnemonic starts with `opcode_prefix` to a non-matrix reader of its result, where one exists within `limit`."""
    def ws(i):
        m = re.match(r"s_nop (\d+)", ins[i])
        return int(m.group(1)) + 1 if m else 1

    found = []
    for i, t in enumerate(ins):
        if not t.startswith(opcode_prefix):
            continue
        dst = _regs(t.split(None, 1)[1].split(",")[0])
        best = None
        stack, seen = [(i + 1, 0)], {}
        while stack:
            j, w = stack.pop()
            while j < len(ins) and w < limit:
                if j in seen and seen[j] <= w:
                    break
                seen[j] = w
                u = ins[j]
                ops = u.split(None, 1)
                allr = _regs(ops[1]) if len(ops) > 1 else set()
                is_store = re.match(r"(ds_write|global_store|buffer_store|flat_store|scratch_store)", u) is not None
                srcs = allr if is_store or len(ops) < 2 else _regs(",".join(ops[1].split(",")[1:]))
                if u.startswith("v_mfma"):
                    if allr & dst:
                        break                     # accumulated into again or fed on: that instruction's own business
                elif srcs & dst and not u.startswith("s_"):
                    if best is None or w < best[0]:
                        best = (w, t, u)
                    break
                elif allr & dst and not u.startswith("s_"):
                    break                         # overwritten: the value is dead on this path
                if u.startswith("s_endpgm"):
                    break
                mb = re.match(r"s_(c?branch\S*)\s+(\S+)", u)
                if mb:
                    tgt = labels.get(mb.group(2))
                    if tgt is not None:
                        stack.append((tgt, w + 1))
                    if mb.group(1) == "branch":
                        break
                w += ws(j)
                j += 1
        if best is not None:
            found.append(best)
    return found
