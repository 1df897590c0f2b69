"""Build checks on the generated assembly: (1) wave-uniform conditions that the compiler re-derived with a
vector compare inside a loop and then reads outside that loop; (2) per-peer write-through stores that each
wait for all memory operations (see serialised_store_findings).

(1):

hipcc keeps a wave-uniform boolean (rank == j, j < n) as a 64-bit lane mask.  Where it needs
the negation it may emit `v_cndmask_b32 v, 0, 1, mask` + `v_cmp_ne_u32 s[a:b], 1, v`; a vector
compare writes bits only for the lanes active at that point.  Inside a loop that lanes leave at
different iterations this gives a mask that is wrong for every lane that has already left, and
code after the loop (a later loop over the same data, say) that tests it can take the wrong side.
The kernels avoid the pattern by forming such conditions from per-lane copies of the rank and the
rank count (`per_lane` in csrc/msx_device.hpp); this module compiles the device code to assembly
and reports any place where the pattern is back.

    python tests/codegen_audit.py          # prints findings, exit status 1 if any
"""
import os
import re
import subprocess
import sys
import tempfile

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2504_09014_amd import build as _build  # noqa: E402

# The instruction idioms searched for below are what THIS compiler emits; another version may lower the same
# source differently, and the scan would then pass without having looked at anything.
VALIDATED_COMPILER = "roc-7.2.0"


def compiler_version():
    """The hipcc banner (its clang line names the ROCm release the compiler was built from)."""
    return subprocess.run([_build.HIPCC, "--version"], capture_output=True, text=True, check=True).stdout

_RE_FN = re.compile(r'^(_Z\w+):')
_RE_LABEL = re.compile(r'^(?:\.L(BB\d+_\d+):|; %bb\.(\d+):)')
_RE_ROUNDTRIP = re.compile(r'v_cmp_ne_u32_e64 (s\[\d+:\d+\]), 1, v\d+')


def device_assembly(out_path):
    """Compile csrc/*.hip for gfx950, device side only, to assembly text."""
    flags = [f for f in _build.FLAGS if f not in ("-shared", "-fPIC")]
    jobs = []
    for k, src in enumerate(_build.sources()):              # one translation unit each, all at once
        part = f"{out_path}.{k}"
        cmd = [_build.HIPCC] + flags + ["--cuda-device-only", "-S", "-o", part, src]
        jobs.append((cmd, part, subprocess.Popen(cmd, stderr=subprocess.DEVNULL)))
    with open(out_path, "w") as out:
        for cmd, part, proc in jobs:
            if proc.wait() != 0:
                raise subprocess.CalledProcessError(proc.returncode, cmd)
            with open(part) as f:
                out.write(f.read())
            os.remove(part)
    return out_path


def _regs(tok):
    m = re.match(r's\[(\d+):(\d+)\]', tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r's(\d+)$', tok)
    if m:
        return {int(m.group(1))}
    return {106, 107} if tok == "vcc" else set()


def parse(path):
    """-> {function: [(block label, innermost loop header or None, instruction), ...]}, parents."""
    funcs, parents = {}, {}
    fn, cur = None, None
    for raw in open(path):
        line = raw.rstrip("\n")
        m = _RE_FN.match(line)
        if m:
            fn = m.group(1)
            cur = ["entry", None]
            funcs[fn] = []
            continue
        if fn is None:
            continue
        if line.startswith("\t.end_amdhsa_kernel") or line.startswith(".Lfunc_end"):
            fn = None
            continue
        m = _RE_LABEL.match(line)
        if m:
            label = m.group(1) or ("bb." + m.group(2))
            loop = None
            mm = re.search(r'in Loop: Header=(BB\d+_\d+) Depth=', line)
            if mm:
                loop = mm.group(1)
            if "Loop Header" in line:
                loop = label
            cur = [label, loop]
            mm = re.search(r'Parent Loop (BB\d+_\d+) Depth', line)    # the outermost parent shares the label's line
            if mm:
                parents.setdefault((fn, label), []).append(mm.group(1))
            continue
        if re.match(r'^\s+;', line):            # further comment lines of a loop header block
            if "Loop Header" in line:
                cur[1] = cur[0]
            mm = re.search(r'Parent Loop (BB\d+_\d+) Depth', line)
            if mm:
                parents.setdefault((fn, cur[0]), []).append(mm.group(1))
            continue
        if line.startswith("\t") and not line.startswith("\t."):
            funcs[fn].append((cur[0], cur[1], line.strip()))
    return funcs, parents


def _chain(parents, fn, loop):
    out = []
    while loop and loop not in out:
        out.append(loop)
        ps = parents.get((fn, loop), [])
        loop = ps[-1] if ps else None           # the innermost parent is listed last
    return out


def findings(path):
    """[(function, (def block, loop, instruction), (use block, loop, instruction)), ...]"""
    funcs, parents = parse(path)
    found = []
    for fn, flat in funcs.items():
        for i, (lab, loop, ins) in enumerate(flat):
            m = _RE_ROUNDTRIP.match(ins)
            if not m or loop is None:
                continue
            d = _regs(m.group(1))
            for lab2, loop2, ins2 in flat[i + 1:]:
                ops = re.split(r'[ ,]+', ins2)
                if ops[0].startswith(("s_cbranch", "s_branch")) or len(ops) < 2:
                    continue
                if any(_regs(t) & d for t in ops[2:]) and loop not in _chain(parents, fn, loop2):
                    found.append((fn, (lab, loop, ins), (lab2, loop2, ins2)))
                    break
                if _regs(ops[1]) & d and not ops[0].startswith(("buffer_store", "global_store")):
                    break                        # redefined
    return found


def serialised_store_findings(path, limit=3):
    """Kernels in which more than `limit` write-through 16-byte stores (or, in kernels with hundreds of
    them, more than one in 64) each sit right behind a full `s_waitcnt vmcnt(0)`.  A serialised per-peer
    sequence shows as one store in eight or more; the first store behind a barrier's own drain, once per
    code path, is not it.

    The write-through stores are inline assembly, so the compiler does not know they are in flight.  When a
    conditional store is the first use of a loaded register it waits for ALL memory operations there, which
    also drains the stores already issued: a sequence of per-peer stores then runs one round trip at a time
    (`settle()` in csrc/msx_device.hpp consumes the loaded vector once, before the stores).  The LL packet
    stores are builtins, which the compiler counts, but across the per-peer conditions it falls back to the
    same full wait: they are checked too (the first phase of 2PA-LL ran seven store round trips in a row).
    -> [(function, stores behind a full wait, write-through stores)]"""
    found = []
    fn, prev, stores, waited = None, [], 0, 0
    for raw in open(path):
        m = _RE_FN.match(raw)
        if m:
            fn, prev, stores, waited = m.group(1), [], 0, 0
            continue
        if fn is None:
            continue
        t = raw.strip()
        if t.startswith(".end_amdhsa_kernel") or t.startswith(".Lfunc_end"):
            if waited > max(limit, stores // 64):
                found.append((fn, waited, stores))
            fn = None
            continue
        if not t or t.startswith(";") or t.startswith("."):
            continue
        # write-through puts, and the LL packet stores (a packet store sits up to eight instructions behind its
        # wait: the four moves that assemble {w0, flag, w1, flag} and the descriptor set-up come in between)
        put = t.startswith("global_store_dwordx4") and " sc1" in t
        packet = t.startswith("buffer_store_dwordx4") and " sc1" in t
        if put or packet:
            stores += 1
            if any(p.startswith("s_waitcnt") and "vmcnt(0)" in p for p in prev[-(3 if put else 8):]):
                waited += 1
        prev.append(t)
    return found


def main():
    with tempfile.TemporaryDirectory() as tmp:
        path = device_assembly(os.path.join(tmp, "msx_device.s"))
        found = findings(path)
        slow = serialised_store_findings(path)
    for fn, d, u in found:
        print(f"{fn}\n   def  [{d[0]} in loop {d[1]}] {d[2]}\n   use  [{u[0]} in loop {u[1]}] {u[2]}")
    for fn, waited, stores in slow:
        print(f"{fn}: {waited} of {stores} write-through stores wait for all memory operations first")
    print(f"{len(found)} lane-mask finding(s), {len(slow)} kernel(s) with serialised stores")
    return 1 if found or slow else 0


if __name__ == "__main__":
    sys.exit(main())
