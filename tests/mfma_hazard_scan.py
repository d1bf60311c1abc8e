"""Static check of the compiled kernels: a vector, LDS or memory instruction that reads the result registers of an
MFMA needs a number of idle issue states after it (more for MFMAs with more passes).  The compiler counts them inside a
basic block but has been seen not to look through a branch that follows the MFMA, so a reader at the head of the branch
target can run too early and see registers the matrix core has not written yet (the decode kernel showed run-to-run
differences in the last bits before idle states were written by hand behind its score MFMAs).  This scan walks the
assembly of a kernel, follows branches behind every MFMA and reports readers that come within `need` issue states."""
import re


def _regs(tok):
    tok = tok.split()[0] if tok.split() else tok
    m = re.match(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def scan(asm_text: str, kernel: str, need: int = 12, horizon: int = 24):
    """Readers of MFMA results reached through at least one branch with fewer than `need` issue states in between."""
    lines = [l.rstrip() for l in asm_text.split("\n")]
    start = [i for i, l in enumerate(lines) if re.match(r"^_Z.*" + kernel + ".*:", l)][0]
    end = [i for i, l in enumerate(lines) if i > start and ".end_amdhsa_kernel" in l][0]
    body = [l for l in lines[start:end] if l.strip() and not l.strip().startswith(";")]
    labels = {}
    for i, l in enumerate(body):
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    is_instr = lambda l: l.startswith("\t") and not l.strip().startswith(".")
    states = lambda x: int(x.split()[1]) + 1 if x.split()[0] == "s_nop" else 1
    found = []
    for i, l in enumerate(body):
        if "v_mfma" not in l:
            continue
        dst = _regs(l.split(None, 1)[1].split(",")[0].strip())
        seen = set()

        def walk(j, left, path):
            while left > 0 and j < len(body):
                x = body[j]
                if not is_instr(x):
                    j += 1
                    continue
                name = x.split()[0]
                if name.startswith("s_cbranch") or name == "s_branch":
                    tgt = x.split()[1]
                    if tgt in labels and (tgt, left) not in seen:
                        seen.add((tgt, left))
                        walk(labels[tgt] + 1, left - 1, path + [tgt])
                    if name == "s_branch":
                        return
                elif "v_mfma" in x:
                    if _regs(x.split(None, 1)[1].split(",")[0].strip()) & dst:
                        return            # accumulating on: the matrix core orders these itself
                elif name.startswith(("v_", "ds_", "global_", "buffer_")):
                    rest = x.split(None, 1)[1] if len(x.split(None, 1)) > 1 else ""
                    toks = [t.strip() for t in rest.split(",")]
                    first_src = 0 if name.startswith(("ds_write", "global_store", "buffer_store")) else 1
                    src = set()
                    for t in toks[first_src:]:
                        src |= _regs(t)
                    if src & dst:
                        if path and horizon - left < need:
                            found.append((l.strip(), path, x.strip(), horizon - left))
                        return
                left -= states(x)
                j += 1

        walk(i + 1, horizon, [])
    return found
