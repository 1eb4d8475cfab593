"""The written-out wait counts of the matrix-core expert kernel, checked against the code the
compiler produced.

The kernel copies token tiles global -> LDS with instructions the compiler does not track and
orders them with ``s_waitcnt vmcnt(N)`` written next to every barrier.  Vector-memory
instructions of a wavefront complete in issue order, so the wait guarantees "every copy but the
most recent group of kNP has landed" exactly when at least N vector-memory instructions were
issued after the last copy of the second most recent group.  Part of those N are weight loads
whose position the compiler chooses, so the property is verified here, on the assembly text the
device object is assembled from, at every such wait of every instantiation and along every path
that reaches it.  No GPU needed.
"""
import os
import re
import subprocess

import pytest

from paper_2505_06481_amd import build as mbuild

SRC = os.path.join(mbuild.CSRC, "ffn_tiled.hip")

VM_PREFIXES = ("global_load", "global_store", "global_atomic", "buffer_load", "buffer_store", "buffer_atomic",
               "flat_load", "flat_store", "flat_atomic", "scratch_load", "scratch_store")
COPY = "global_load_lds_dwordx4"


def device_assembly():
    """Assembly of ffn_tiled.hip for gfx950: the file the in-tree build left behind if it is
    newer than the source, otherwise a fresh compile with the same flags."""
    deps = [SRC] + mbuild._headers()
    if os.path.exists(mbuild.TILED_ASM) and os.path.getmtime(mbuild.TILED_ASM) >= max(map(os.path.getmtime, deps)):
        return open(mbuild.TILED_ASM).read()
    os.makedirs(mbuild.OBJ_DIR, exist_ok=True)
    out = os.path.join(mbuild.OBJ_DIR, "ffn_tiled_check.s")
    subprocess.run([mbuild.HIPCC] + mbuild.FLAGS + ["--cuda-device-only", "-S", SRC, "-o", out], check=True,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return open(out).read()


class Func:
    """Basic blocks of one function: instruction lists, successor and predecessor edges."""

    def __init__(self, name, lines):
        self.name = name
        self.blocks = []     # list of instruction lists
        label_at = {}        # label -> block index
        cur = []
        self.blocks.append(cur)
        for ln in lines:
            ln = ln.split(";")[0].rstrip()
            if not ln.strip():
                continue
            m = re.match(r"^(\.LBB\w+):", ln)
            if m:
                if cur:
                    cur = []
                    self.blocks.append(cur)
                label_at[m.group(1)] = len(self.blocks) - 1
                continue
            if not ln.startswith("\t") or ln.lstrip().startswith("."):
                continue
            ins = ln.strip()
            cur.append(ins)
            if ins.startswith(("s_branch", "s_cbranch", "s_endpgm")):
                cur = []
                self.blocks.append(cur)
        self.succ = [[] for _ in self.blocks]
        for b, ins_list in enumerate(self.blocks):
            last = ins_list[-1] if ins_list else ""
            if last.startswith("s_endpgm"):
                continue
            if last.startswith(("s_branch", "s_cbranch")):
                self.succ[b].append(label_at[last.split()[-1]])
                if last.startswith("s_branch"):
                    continue
            if b + 1 < len(self.blocks):
                self.succ[b].append(b + 1)
        self.pred = [[] for _ in self.blocks]
        for b, ss in enumerate(self.succ):
            for t in ss:
                self.pred[t].append(b)


def functions(text, prefix):
    out = []
    for m in re.finditer(r"^(%s\w*):.*?^\.Lfunc_end\d+:" % re.escape(prefix), text, re.S | re.M):
        out.append(Func(m.group(1), m.group(0).splitlines()[1:]))
    return out


def wait_sites(fn):
    """(block, index, N) of every written-out "s_waitcnt vmcnt(N) ... ; s_barrier" pair."""
    sites = []
    for b, ins_list in enumerate(fn.blocks):
        for i, ins in enumerate(ins_list[:-1]):
            m = re.match(r"s_waitcnt\b.*\bvmcnt\((\d+)\)", ins)
            if m and ins_list[i + 1].startswith("s_barrier"):
                sites.append((b, i, int(m.group(1))))
    return sites


def min_issued_since_older_copies(fn, block, index, knp):
    """Over every path that reaches the wait: the number of vector-memory instructions issued
    after the last copy of the second most recent copy group (= before the (knp+1)-th copy, walking
    backwards).  Returns the minimum, or None if some path reaches the function entry first."""
    best = [None]
    seen = set()
    stack = [(block, index, 0, 0)]   # block, instructions of it still to scan, copies seen, vm ops seen
    while stack:
        b, n, copies, vm = stack.pop()
        done = False
        for ins in reversed(fn.blocks[b][:n]):
            if ins.startswith(VM_PREFIXES):
                if ins.startswith(COPY):
                    copies += 1
                    if copies == knp + 1:
                        best[0] = vm if best[0] is None else min(best[0], vm)
                        done = True
                        break
                vm += 1
        if done:
            continue
        if not fn.pred[b]:
            return None
        for p in fn.pred[b]:
            key = (p, copies, vm)
            if key not in seen:
                seen.add(key)
                stack.append((p, len(fn.blocks[p]), copies, vm))
    return best[0]


def check_function(fn, knp):
    """List of (N, issued) for every written-out wait; raises on a violated one."""
    res = []
    for b, i, n in wait_sites(fn):
        issued = min_issued_since_older_copies(fn, b, i, knp)
        assert issued is not None, f"{fn.name}: a path reaches the wait before {knp + 1} copies were issued"
        assert issued >= n, (f"{fn.name}: s_waitcnt vmcnt({n}) is preceded by only {issued} vector-memory "
                             f"instructions since the older copy groups: an older copy could still be in flight")
        res.append((n, issued))
    return res


def test_checker_flags_a_short_window():
    """The checker itself: a hand-written stream in which a weight load has been moved from behind
    the copies to in front of them must be refused, the original accepted."""
    def stream(loads_after):
        body = ["\tglobal_load_lds_dwordx4 v1, s[0:1]"] * 2                     # older group (knp = 2)
        body += ["\tglobal_load_dwordx4 v[2:5], v[6:7], off"] * (3 - loads_after)
        body += ["\tglobal_load_lds_dwordx4 v1, s[0:1]"] * 2                    # older group
        body += ["\tglobal_load_dwordx4 v[2:5], v[6:7], off"] * loads_after
        body += ["\tglobal_load_lds_dwordx4 v1, s[0:1]"] * 2                    # most recent group
        body += ["\ts_waitcnt vmcnt(5)", "\ts_barrier", "\ts_endpgm"]
        return Func("f", body)
    assert check_function(stream(3), knp=2) == [(5, 5)]
    with pytest.raises(AssertionError):
        check_function(stream(2), knp=2)
    # a loop: the window wraps around the back edge
    loop = Func("g", ["\tglobal_load_lds_dwordx4 v1, s[0:1]", ".LBB9_1:",
                      "\tglobal_load_dwordx4 v[2:5], v[6:7], off", "\ts_waitcnt vmcnt(2)", "\ts_barrier",
                      "\tglobal_load_lds_dwordx4 v1, s[0:1]", "\ts_cbranch_scc1 .LBB9_1", "\ts_endpgm"])
    with pytest.raises(AssertionError):     # first trip: only one copy precedes the wait
        check_function(loop, knp=1)


def test_every_written_out_wait_of_the_tiled_kernel_is_covered():
    text = device_assembly()
    fns = functions(text, "_ZN4mmoe12tiled_kernel")
    # 4 products (three activations, down) x 2 tile heights, and the three products without a gate
    # once more with one weight block per wavefront (128-row tiles only)
    assert len(fns) == 14, [f.name for f in fns]
    for fn in fns:
        bm, nb = (int(x) for x in re.search(r"ILi\d+ELi(\d+)ELi(\d+)EE", fn.name).groups())
        knp = bm * 8 // 256                               # copies per wavefront and step
        nj_variants, steps_per_trip = bm // 32 if bm == 256 else 4, (16 if bm == 256 or nb == 1 else 8) // 4
        res = check_function(fn, knp)
        # one wait in the prologue and one per unrolled step of the main loop, per instantiation
        assert len(res) == nj_variants * (1 + steps_per_trip), (fn.name, len(res))
        print(f"{fn.name}: {len(res)} waits, smallest margin {min(i - n for n, i in res)}")
