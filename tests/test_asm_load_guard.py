"""Host-side guard for inline-assembly memory loads in the HIP sources.

A vector-memory load issued from inline assembly returns its data long after the asm statement has "executed"
as far as the compiler can tell.  If the destination is a write-only operand ("=v") that nothing reads, the
register is dead at once, the allocator reuses it, and the late return overwrites whatever lives there by then
(a loop index, an address).  The rule the sources must keep: a load with a register destination names it as a
read-write operand ("+v"), and the same variable passes through an empty asm fence (asm volatile("" : "+v"(x)))
after the wait that covers the load, so that the register holds nothing else in between.  Loads that deliver
straight into LDS have no register destination and must not declare one.  CPU only: it reads the sources.
"""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_14376_amd", "csrc")

# (no leading \b: in the source text an instruction often follows the two characters of a "\t" escape)
LOAD = re.compile(r"(global_load|buffer_load|flat_load|scratch_load)_\w+")


def _asm_statements(text):
    """(start offset, body) of every asm statement, body = the text between its outer parentheses."""
    out = []
    for m in re.finditer(r"\basm\s+(?:volatile\s*)?\(", text):
        depth, i = 1, m.end()
        while depth and i < len(text):
            depth += {"(": 1, ")": -1}.get(text[i], 0)
            i += 1
        out.append((m.start(), text[m.end():i - 1]))
    return out


def _split_sections(body):
    """template, outputs, inputs, clobbers: split at the colons outside string literals and parentheses."""
    parts, cur, depth, in_str, i = [], [], 0, False, 0
    while i < len(body):
        c = body[i]
        if in_str:
            cur.append(c)
            if c == "\\":
                cur.append(body[i + 1]); i += 1
            elif c == '"':
                in_str = False
        elif c == '"':
            in_str = True; cur.append(c)
        elif c in "([":
            depth += 1; cur.append(c)
        elif c in ")]":
            depth -= 1; cur.append(c)
        elif c == ":" and depth == 0:
            if body[i:i + 2] == "::":
                parts.append("".join(cur)); parts.append(""); cur = []; i += 1
            else:
                parts.append("".join(cur)); cur = []
        else:
            cur.append(c)
        i += 1
    parts.append("".join(cur))
    return (parts + ["", "", ""])[:4]


def _operands(section):
    return re.findall(r'"([^"]*)"\s*\(\s*([^()]+(?:\([^()]*\))?[^()]*)\)', section)


def check_source(text):
    """list of violations (strings) in one source text"""
    bad = []
    stmts = _asm_statements(text)
    fences = []   # (offset, variable) of empty-template fences with a "+v" operand
    for off, body in stmts:
        tmpl, outs, _, _ = _split_sections(body)
        if re.sub(r'["\s]', "", tmpl) == "":
            for cons, var in _operands(outs):
                if cons == "+v":
                    fences.append((off, var.strip()))
    for off, body in stmts:
        tmpl, outs, _, _ = _split_sections(body)
        if not LOAD.search(tmpl):
            continue
        line = text.count("\n", 0, off) + 1
        to_lds = "_lds_" in tmpl or re.search(r"\blds\b", tmpl) is not None
        ops = _operands(outs)
        if to_lds:
            if ops:
                bad.append("line %d: a load into LDS declares a register output" % line)
            continue
        if not ops:
            bad.append("line %d: a register load without a declared destination operand" % line)
        for cons, var in ops:
            if cons != "+v":
                bad.append("line %d: destination operand %r(%s) must be \"+v\"" % (line, cons, var.strip()))
            elif not any(o > off and v == var.strip() for o, v in fences):
                bad.append("line %d: destination %s is not kept live by a later asm fence" % (line, var.strip()))
    return bad


def test_no_asm_load_with_a_dead_destination():
    files = sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(CSRC, "*.hip")))
    assert files
    problems = []
    for path in files:
        problems += ["%s %s" % (os.path.basename(path), p) for p in check_source(open(path).read())]
    assert not problems, "\n".join(problems)


def test_the_guard_sees_the_fault_class():
    """the checker itself: the pattern that faulted is flagged, the safe forms pass"""
    write_only = 'asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(r) : "v"(off), "s"(base) : "memory");'
    assert check_source(write_only)
    unfenced = 'asm volatile("global_load_dword %0, %1, %2" : "+v"(r) : "v"(off), "s"(base));'
    assert check_source(unfenced)
    fenced = unfenced + '\nasm volatile("s_waitcnt vmcnt(0)" ::: "memory");\nasm volatile("" : "+v"(r));'
    assert not check_source(fenced)
    to_lds = 'asm volatile("s_mov_b32 m0, %0\\n\\tglobal_load_lds_dwordx4 %1, %2" :: "s"(la), "v"(voff), "s"(gu) : "memory", "m0");'
    assert not check_source(to_lds)
    assert check_source(to_lds.replace('::', ': "=v"(x) :', 1))
