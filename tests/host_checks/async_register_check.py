"""Flow check on the compiled fused GEMM kernel (gfx950 assembly text on stdin or in the file named by argv[1]).

The kernel issues its row loads (buffer_load_dwordx2 / buffer_load_dword into registers) and its table lookups
(ds_bpermute_b32) as volatile asm and waits for them by hand.  The compiler takes an asm's outputs as written when the
statement ends, so nothing but the hand-placed order keeps it from reading, copying or reusing such a register while
the data is still on its way.  This script walks every basic block of the kernel that holds MFMAs (the main loop, twice
to cover its back edge, and its peeled iterations) and reports any instruction that touches a register
between its asynchronous write and the next wait that covers it (any s_waitcnt with vmcnt for the loads, an
s_waitcnt lgkmcnt(0) for the lookups and fragment reads)."""
import re
import sys

KERNEL = "gemm_nt_kernelILi256ELi4ELb1EE"


def regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def check(text, kernel=KERNEL):
    start = [m.start() for m in re.finditer(r"^_ZN\S*" + kernel + r"\S*:", text, re.M)]
    if not start:
        return ["kernel not found"], 0
    body = text[start[0]:text.index("s_endpgm", start[0])]
    lines = [l.strip() for l in body.split("\n") if l.strip() and not l.strip().startswith(";")]
    blocks, cur, name = [], [], "entry"
    for l in lines:
        if l.startswith(".LBB"):
            blocks.append((name, cur))
            cur, name = [], l.split(":")[0]
        elif not l.startswith(".") and not l.endswith(":"):
            cur.append(l)
    blocks.append((name, cur))
    bad, seen = [], 0
    for name, b in blocks:
        if not any(x.startswith("v_mfma") for x in b):
            continue
        seen += 1
        # the hardware's two counters, as queues of the destination registers of the operations in flight: memory
        # operations return in order, and s_waitcnt vmcnt(N) / lgkmcnt(N) waits until at most N are outstanding
        vm, lg = [], []
        # a block that branches back to itself is scanned twice, reporting on the second pass (what is in flight at
        # its end is in flight at its start); any other block starts behind the waits of the block before it
        loop = any(x.startswith("s_cbranch") and x.split()[-1] == name for x in b)
        for rnd in ((0, 1) if loop else (1,)):
            for l in b:
                parts = l.replace(",", " ").split()
                op, ops = parts[0], parts[1:]
                if op == "s_waitcnt":
                    m = re.search(r"vmcnt\((\d+)\)", l)
                    if m:
                        del vm[:max(0, len(vm) - int(m.group(1)))]
                    m = re.search(r"lgkmcnt\((\d+)\)", l)
                    if m:
                        del lg[:max(0, len(lg) - int(m.group(1)))]
                    continue
                if not ops:
                    continue
                d, srcs = regs(ops[0]), set()
                for t in ops[1:]:
                    srcs |= regs(t)
                store = op.startswith("ds_write") or "store" in op
                if store:
                    srcs |= d
                    d = set()
                flying = set().union(*vm, *lg) if (vm or lg) else set()
                if rnd == 1 and (srcs | d) & flying:
                    bad.append(l)
                if op.startswith("buffer_") or op.startswith("global_") or op.startswith("scratch_"):
                    vm.append(set() if (store or " lds" in l) else d)
                elif op.startswith("ds_"):
                    lg.append(d)
                elif op.startswith("s_load") or op.startswith("s_buffer_load"):
                    lg.append(set())                          # scalar loads share the counter (and return out of order:
                                                              # the compiler waits for them with lgkmcnt(0))
    return bad, seen


if __name__ == "__main__":
    text = open(sys.argv[1]).read() if len(sys.argv) > 1 else sys.stdin.read()
    bad, seen = check(text)
    if bad or seen < 5:
        print("FAIL", seen, len(bad))
        for l in bad[:20]:
            print("  ", l)
        sys.exit(1)
    print("OK", seen, "blocks")
