"""Build-time check of the generated kernels: no instruction may touch a register that an
LDS read issued from inline assembly is still filling.

The GEMM and attention main loops issue their LDS fragment reads as inline ``ds_read`` and wait
for them later with a counted ``s_waitcnt lgkmcnt(N)``, so that reads, direct-to-LDS loads and
MFMAs overlap.  The compiler does not know that the destination registers of such a read are
not valid until that wait; it is kept from using them early by operand ties placed behind the
wait.  Nothing in the language stops it from inserting a register copy in between, though, and
a copy that reads an in-flight register silently corrupts a fragment.  This module therefore
reads the assembly hipcc produces for the kernels (its own output, ``-S``) and proves, by a
forward data-flow over each kernel's control-flow graph, that no register copy or spill reads a
register a pending ``ds_read`` is still to write.  build() runs it and fails loudly otherwise.

Model: LGKM operations (LDS accesses, scalar memory loads) enter a queue in program order; LDS
operations complete in order, so ``lgkmcnt(N)`` retires the oldest LDS entries beyond the
youngest N (scalar loads may complete out of order: each one in the queue is assumed to have
taken one of the completions the wait guarantees).  Where paths with different queues meet they
are aligned at the youngest entry and united position by position.  Queues are cut to the 16
operations the hardware counter can hold.  A register that a later instruction overwrites leaves
the pending sets (reads pending only on paths no execution takes must not taint the registers'
next values) -- except where the read was issued in the same basic block: that overwrite is on a
real path, the LDS return would clobber the new value, and it is reported.
"""

from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from typing import Dict, List, Optional, Tuple

# the LGKM counter of this hardware family has 4 bits: a wave cannot have more operations
# outstanding, so anything older than the youngest 16 has completed (this also bounds the
# data-flow: queues cannot grow around loops)
_MAX_OUTSTANDING = 16

# What is checked: instructions by which the compiler moves a value it believes to be ready --
# register copies and spills.  (Checking every use would need the branch conditions: the walk is
# path-insensitive, and e.g. "fragments requested at a stage hand-over, then loop exit" is a path
# of the graph that no execution takes.)
_COPY_OPS = ("v_mov_b32", "v_mov_b64", "v_pk_mov", "v_swap", "v_accvgpr_write", "scratch_store")

_REG = re.compile(r"\b([va])(\d+)\b|\b([va])\[(\d+):(\d+)\]")
_LABEL = re.compile(r"^([.\w$]+):")


def _regs(text: str):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(3), i) for i in range(int(m.group(4)), int(m.group(5)) + 1))
    return frozenset(out)


class Inst:
    __slots__ = ("line", "op", "dst", "src", "text")

    def __init__(self, line: int, text: str):
        self.line, self.text = line, text
        parts = text.split(None, 1)
        self.op = parts[0]
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        writes_first = self.op.startswith(("v_", "ds_read", "ds_bpermute", "ds_permute", "global_load", "buffer_load",
                                           "scratch_load", "flat_load")) and not self.op.startswith("global_load_lds")
        if self.op.startswith(("v_cmp", "v_cmpx")) or not ops:
            writes_first = False
        self.dst = _regs(ops[0]) if writes_first else frozenset()
        self.src = _regs(",".join(ops[1:] if writes_first else ops))
        if self.op.startswith("v_mfma") or self.op.startswith("v_fmac") or self.op.startswith("v_mac"):
            self.src = self.src | self.dst          # accumulating forms read their destination


def _is_lgkm(op: str) -> bool:
    return op.startswith(("ds_", "s_load", "s_buffer_load", "s_memtime", "s_memrealtime", "s_sendmsg"))


def _wait_count(text: str) -> Optional[int]:
    m = re.search(r"lgkmcnt\((\d+)\)", text)
    return int(m.group(1)) if m else None


def _functions(asm: str):
    lines = asm.split("\n")
    i = 0
    while i < len(lines):
        m = re.match(r"^(\w+):\s*(;.*)?$", lines[i])
        if m and i > 0 and ".type" in "".join(lines[max(0, i - 6):i]) and "@function" in "".join(lines[max(0, i - 6):i]):
            name = m.group(1)
            j = i + 1
            while j < len(lines) and not lines[j].startswith(".Lfunc_end"):
                j += 1
            yield name, i, lines[i + 1:j]
            i = j
        i += 1


def check_function(name: str, first_line: int, body: List[str]) -> List[str]:
    # ---- basic blocks
    blocks: List[Dict] = [{"label": None, "insts": [], "succ": []}]
    label_of: Dict[str, int] = {}
    for k, raw in enumerate(body):
        t = raw.split(";")[0].strip()
        if not t:
            continue
        lm = _LABEL.match(t)
        if lm:
            if blocks[-1]["insts"] or blocks[-1]["label"] is not None:
                blocks.append({"label": lm.group(1), "insts": [], "succ": []})
            else:
                blocks[-1]["label"] = lm.group(1)
            label_of[lm.group(1)] = len(blocks) - 1
            continue
        if t.startswith("."):
            continue
        blocks[-1]["insts"].append(Inst(first_line + 1 + k, t))
        if t.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc")):
            blocks.append({"label": None, "insts": [], "succ": []})
    for bi, b in enumerate(blocks):
        last = b["insts"][-1] if b["insts"] else None
        fall = True
        if last is not None:
            if last.op.startswith("s_cbranch") or last.op == "s_branch":
                tgt = last.text.split()[-1]
                if tgt in label_of:
                    b["succ"].append(label_of[tgt])
                fall = last.op != "s_branch"
            if last.op.startswith(("s_endpgm", "s_setpc")):
                fall = False
        if fall and bi + 1 < len(blocks):
            b["succ"].append(bi + 1)

    # ---- data-flow.  State = queue of pending LGKM operations, oldest first.
    Entry = tuple          # of frozenset (registers an LDS operation will write) or "smem"
    state_in: Dict[int, Entry] = {0: ()}
    work = [0]
    errors: List[str] = []
    seen_err = set()

    def merge(a: Entry, b: Entry) -> Entry:
        # both are in-order queues: align them at the youngest entry and unite position by
        # position (older entries of the longer one are kept) -- what lgkmcnt(N) keeps, the
        # youngest N, is then a superset of what either path keeps
        if a == b:
            return a
        lo, hi = (a, b) if len(a) <= len(b) else (b, a)
        head = hi[:len(hi) - len(lo)]
        tail = tuple(("smem" if "smem" in (x, y) else x | y) for x, y in zip(hi[len(hi) - len(lo):], lo))
        return head + tail

    while work:
        bi = work.pop()
        q = list(state_in[bi])
        local = 0            # the youngest `local` entries of q were issued in this very block
        for ins in blocks[bi]["insts"]:
            pending = frozenset().union(*[e for e in q if e != "smem"]) if q else frozenset()
            touched = ins.src & pending if ins.op.startswith(_COPY_OPS) else frozenset()
            if touched and (ins.line, ins.text) not in seen_err:
                seen_err.add((ins.line, ins.text))
                regs = ", ".join("%s%d" % r for r in sorted(touched)[:6])
                errors.append("%s: asm line %d: `%s` copies %s while an LDS read into it may be pending"
                              % (name, ins.line, ins.text, regs))
            n = _wait_count(ins.text) if ins.op == "s_waitcnt" else None
            if n is not None:
                if n == 0:
                    q = []
                else:
                    # scalar loads may complete before older LDS operations: of the len(q) - n
                    # completions the wait guarantees, up to k may be theirs
                    k = sum(1 for e in q if e == "smem")
                    r = max(0, len(q) - n - k)
                    kept = []
                    for e in q:
                        if e != "smem" and r > 0:
                            r -= 1
                        else:
                            kept.append(e)
                    q = kept
                local = min(local, len(q))
            if ins.dst and local and not ins.op.startswith(("ds_read", "ds_bpermute", "ds_permute")):
                # an overwrite of a register whose read was issued in this same block and is
                # still pending is on a path that is certainly taken: the LDS return would land
                # on top of the new value
                mine = frozenset().union(*[e for e in q[len(q) - local:] if e != "smem"])
                hit = ins.dst & mine
                if hit and (ins.line, "w") not in seen_err:
                    seen_err.add((ins.line, "w"))
                    regs = ", ".join("%s%d" % r for r in sorted(hit)[:6])
                    errors.append("%s: asm line %d: `%s` overwrites %s while an LDS read into it is in flight"
                                  % (name, ins.line, ins.text, regs))
            if ins.dst and not ins.op.startswith(("ds_read", "ds_bpermute", "ds_permute")) and q:
                # otherwise a register the program overwrites is no longer one a pending read is
                # awaited in (without this, reads that are pending only on a path no execution
                # takes -- requested at a hand-over, then loop exit -- would taint whatever the
                # epilogue keeps in those registers)
                q = [e if e == "smem" else e - ins.dst for e in q]
            if _is_lgkm(ins.op):
                if ins.op.startswith("s_"):
                    q.append("smem")
                else:
                    q.append(ins.dst if ins.op.startswith(("ds_read", "ds_bpermute", "ds_permute")) else frozenset())
                local = min(local + 1, _MAX_OUTSTANDING)
        out: Entry = tuple(q[-_MAX_OUTSTANDING:])
        for s in blocks[bi]["succ"]:
            new = merge(state_in[s], out) if s in state_in else out
            if state_in.get(s) != new:
                state_in[s] = new
                work.append(s)
    return errors


def check_asm(asm: str, only: Tuple[str, ...] = ()) -> List[str]:
    errors: List[str] = []
    n = 0
    for name, first, body in _functions(asm):
        if only and not any(o in name for o in only):
            continue
        n += 1
        errors.extend(check_function(name, first, body))
    if n == 0:
        errors.append("no kernel found in the assembly (wrong file?)")
    return errors


def check_sources(hipcc: str, flags, sources, only=("gemm_bf16_kernel", "attn_bf16_kernel")) -> None:
    """Compile each source to device assembly and run the check; raise on any finding."""
    with tempfile.TemporaryDirectory() as tmp:
        for src in sources:
            out = os.path.join(tmp, os.path.basename(src) + ".s")
            cmd = [hipcc, *[f for f in flags if f != "-fPIC"], "-S", "--cuda-device-only", src, "-o", out]
            r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if r.returncode != 0:
                raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
            errs = check_asm(open(out).read(), only)
            if errs:
                raise RuntimeError("LDS wait check failed for %s:\n  %s" % (src, "\n  ".join(errs[:20])))


if __name__ == "__main__":
    e = check_asm(open(sys.argv[1]).read(), tuple(sys.argv[2:]))
    print("\n".join(e) if e else "ok")
    sys.exit(1 if e else 0)
