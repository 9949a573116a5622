"""A check on emitted gfx950 ISA: after a matrix instruction written as asm with its accumulator in accumulation
registers (the compiler knows nothing of its latency) nothing but a matrix instruction on the same accumulator may
touch those registers until enough wait states have passed.  Follows branches."""
import re

WAIT = 14   # instruction slots (each at least one wait state) that must separate the two, unless s_nops intervene


def parse(text, name_pattern):
    """{kernel symbol: (instructions [(opcode, operands)], {label: index of the instruction it stands in front of})}"""
    out = {}
    for f in re.split(r"\n(?=_Z\w+:)", text)[1:]:
        name = f.split(":")[0]
        if not re.search(name_pattern, name):
            continue
        ins, labels = [], {}
        for line in f.split("\n")[1:]:
            line = line.split(";")[0].rstrip()
            if not line.strip():
                continue
            m = re.match(r"^(\.LBB\w+):", line)
            if m:
                labels[m.group(1)] = len(ins)
                continue
            if line.strip().startswith("."):
                continue
            t = line.strip().split(None, 1)
            ins.append((t[0], t[1] if len(t) > 1 else ""))
            if t[0] == "s_endpgm":
                break
        out[name] = (ins, labels)
    return out


def acc_regs(operands):
    r = set()
    for m in re.finditer(r"\ba\[(\d+):(\d+)\]", operands):
        r.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\ba(\d+)\b", operands):
        r.add(int(m.group(1)))
    return r


def violations(ins, labels):
    bad = []
    for i, (op, args) in enumerate(ins):
        if not op.startswith("v_mfma") or not args.split(",")[0].strip().startswith("a["):
            continue
        d = acc_regs(args.split(",")[0])
        seen, stack = set(), [(i + 1, 0)]
        while stack:
            j, w = stack.pop()
            while j < len(ins) and w < WAIT:
                o, a = ins[j]
                if o == "s_nop":
                    w += int(a.strip(), 0) + 1
                elif o.startswith("v_mfma"):
                    if acc_regs(a.split(",")[0]) == d:
                        break                      # the chain goes on: that instruction is checked on its own
                    if acc_regs(a) & d:
                        bad.append((i, j, ins[i], ins[j]))
                        break
                    w += 4                         # a matrix instruction holds the issue for at least its first passes
                elif acc_regs(a) & d:
                    bad.append((i, j, ins[i], ins[j]))
                    break
                elif o == "s_branch":
                    j = labels.get(a.strip(), len(ins))
                    w += 1
                    continue
                elif o == "s_endpgm":
                    break
                else:
                    if o.startswith("s_cbranch") and a.strip() in labels and (labels[a.strip()], w) not in seen:
                        seen.add((labels[a.strip()], w))
                        stack.append((labels[a.strip()], w + 1))
                    w += 1
                j += 1
    return bad
