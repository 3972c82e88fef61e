"""The hand-over between the chain wave and the weights wave of the two-wave backward kernel
(paper_2404_19760_amd/csrc/lp_mfma_bwd_ws.h), checked on the CPU as a protocol: the sequence of
waits, buffer accesses and counter updates of either role is read from the kernel's source, and
every interleaving of the two sequences over a few steps is explored.  Required: no interleaving
blocks for good, and every read of a shared LDS buffer by the weights wave sees exactly the item
the chain wave wrote for it (nothing is overwritten before, or while, it is read).  Host logic
only; timing, the bounded polling and the LDS ordering of the hardware are not modelled."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2404_19760_amd", "csrc", "lp_mfma_bwd_ws.h")
BUFFERS = ("SLOT0", "SLOT1", "F", "ZO", "DFT", "REC")
STEPS = 4


def _enum(text, name):
    body = re.search(r"enum %s \{([^}]*)\}" % name, text).group(1)
    return [t.strip() for t in body.split(",") if t.strip()]


def _role_ops(lines):
    """[('await', back, stage) | ('post', stage) | ('touch', buffer)] in program order."""
    ops = []
    for line in lines:
        code = line.split("//")[0]
        m = re.search(r"ho\.await\(progress\(n(?: - (\d+))?, (\w+)\)\)", code)
        if m:
            ops.append(("await", int(m.group(1) or 0), m.group(2)))
            continue
        m = re.search(r"ho\.post\(progress\(n, (\w+)\)\)", code)
        if m:
            ops.append(("post", m.group(1)))
            continue
        m = re.search(r"P::(\w+)", code)
        if m and m.group(1) in BUFFERS:
            ops.append(("touch", m.group(1)))
    return ops


def _parse():
    text = open(SRC).read()
    chain_stages, weights_stages = _enum(text, "ChainStage"), _enum(text, "WeightsStage")
    lines = text.split("\n")
    a0 = next(i for i, l in enumerate(lines) if "= chain wave =" in l)
    b0 = next(i for i, l in enumerate(lines) if "= weights wave =" in l)
    b1 = next(i for i, l in enumerate(lines) if "this pair's record of partial sums" in l)
    init = re.search(r"i == 8 \? progress\(0, (\w+)\) : 0", text).group(1)
    # only the loop over the steps: from the first await of a role on
    chain = _role_ops(lines[a0:b0])
    shared = {o[1] for o in chain if o[0] == "touch"}
    weights = []
    since_post = set()   # several accesses of one buffer before the next counter update read the same item
    for o in _role_ops(lines[b0:b1]):
        if o[0] == "post":
            since_post = set()
        if o[0] == "touch":
            if o[1] not in shared or o[1] in since_post:
                continue
            since_post.add(o[1])
        weights.append(o)
    first = lambda ops: next(i for i, o in enumerate(ops) if o[0] == "await")
    return chain[first(chain):], weights[first(weights):], chain_stages, weights_stages, init


def _unroll(ops, steps, reader):
    """The role's operations over `steps` steps, with the step number attached; a read is checked
    where it starts and again right before the counter update that releases the buffer."""
    out = []
    for n in range(1, steps + 1):
        count = {}
        open_reads = []
        for op in ops:
            if op[0] == "await":
                out.append(("await", n - op[1], op[2]))
            elif op[0] == "post":
                out.extend(open_reads)
                open_reads = []
                out.append(("post", n, op[1]))
            else:
                buf = op[1] if op[1] != "REC" else "REC%d" % (n & 1)
                k = count.get(buf, 0)
                count[buf] = k + 1
                item = (buf, n, k)
                if reader:
                    out.append(("read", item))
                    open_reads.append(("read", item))
                else:
                    out.append(("write", item))
        out.extend(open_reads)
    return out


def test_source_declares_the_expected_protocol():
    chain, weights, cs, ws, init = _parse()
    assert len(cs) <= 8 and len(ws) <= 8          # 8 n + stage
    # every stage is posted exactly once per step, in increasing order (the counter never goes back)
    for ops, stages in ((chain, cs), (weights, ws)):
        posted = [o[1] for o in ops if o[0] == "post"]
        assert posted == stages
    # the chain wave only writes the shared buffers, the weights wave only reads them, and every item
    # written in a step is read in that step (a buffer the chain wave never touches is the weights
    # wave's own)
    written = [o[1] for o in chain if o[0] == "touch"]
    read = [o[1] for o in weights if o[0] == "touch" and o[1] in set(written)]
    assert sorted(written) == sorted(read) and {"SLOT0", "SLOT1", "F", "ZO", "REC"} <= set(written)
    assert init == ws[-1]


def test_no_interleaving_deadlocks_or_reads_a_wrong_item():
    chain, weights, cs, ws, init = _parse()
    value = lambda n, stage, stages: 8 * n + stages.index(stage)
    A = _unroll(chain, STEPS, reader=False)
    B = _unroll(weights, STEPS, reader=True)
    # counters and buffer contents are functions of how far each role has got
    def counter(prog, pc, stages, start):
        v = start
        for op in prog[:pc]:
            if op[0] == "post":
                v = value(op[1], op[2], stages)
        return v
    ca = [counter(A, pc, cs, 0) for pc in range(len(A) + 1)]
    cb = [counter(B, pc, ws, value(0, init, ws)) for pc in range(len(B) + 1)]
    contents = [{}]
    for op in A:
        cur = dict(contents[-1])
        if op[0] == "write":
            cur[op[1][0]] = op[1]
        contents.append(cur)

    def can_run(prog, pc, other_counter, other_stages):
        if pc >= len(prog):
            return False
        op = prog[pc]
        return op[0] != "await" or other_counter >= value(op[1], op[2], other_stages)

    seen, stack = set(), [(0, 0)]
    while stack:
        pa, pb = stack.pop()
        if (pa, pb) in seen:
            continue
        seen.add((pa, pb))
        ra = can_run(A, pa, cb[pb], ws)
        rb = can_run(B, pb, ca[pa], cs)
        assert ra or rb or (pa == len(A) and pb == len(B)), \
            f"blocked for good: chain wave at {A[pa] if pa < len(A) else 'end'}, weights wave at {B[pb] if pb < len(B) else 'end'}"
        if ra:
            stack.append((pa + 1, pb))
        if rb:
            op = B[pb]
            if op[0] == "read":
                got = contents[pa].get(op[1][0])
                assert got == op[1], f"the weights wave reads {op[1]} but the buffer holds {got} (chain wave at {pa})"
            stack.append((pa, pb + 1))
    assert (len(A), len(B)) in seen
    assert len(seen) > len(A) + len(B)   # more than one interleaving was explored
