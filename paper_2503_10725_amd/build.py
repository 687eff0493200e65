"""Build step: compile the HIP sources for gfx950.

    python -m paper_2503_10725_amd.build     libssmm.so        the library
                                             libssmm_tune.so   the same sources with -DSSMM_TUNING: its tile and split
                                                               rules read override knobs from the environment (tests
                                                               that force a code path, sweeps on the device; never
                                                               what a user of the library loads)
                                             libssmm_probe.so  bench-only probes (MFMA rate, HBM streaming rate)

Every build of the library also compiles the SSMM kernels to device assembly and checks it: no SSMM
kernel may use scratch memory, no hand-scheduled kernel may hold more accumulation registers than its
accumulators need, and no instruction may touch a register while an asm load into it is in flight.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libssmm.so")
TUNE_LIB = os.path.join(PKG, "libssmm_tune.so")
PROBE_LIB = os.path.join(PKG, "libssmm_probe.so")
OBJ_DIR = os.path.join(PKG, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no packed-fp32 instructions: some forms have returned wrong results on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]
REPORT = "-Rpass-analysis=kernel-resource-usage"   # per-kernel register / scratch report, checked below
INCLUDES = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")]
HAND_SCHEDULED = "ssmm_ffn.hip"   # the source whose kernels issue loads as asm


def hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def sources():
    return sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))


def run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return res.returncode, res.stdout.splitlines()


def build(verbose=True, extra=(), out=LIB):
    """Compile every source of the library in parallel, check the kernels, link `out`."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = "tune_" if out != LIB else ""
    jobs = []
    for src in sources():
        obj = os.path.join(OBJ_DIR, tag + os.path.basename(src) + ".o")
        jobs.append(("obj", src, [hipcc(), *HIPCC_FLAGS, REPORT, *extra, *INCLUDES, "-c", src, "-o", obj], obj))
    asm_path = os.path.join(OBJ_DIR, tag + HAND_SCHEDULED + ".s")
    jobs.append(("asm", HAND_SCHEDULED,
                 [hipcc(), *HIPCC_FLAGS, *extra, *INCLUDES, "--cuda-device-only", "-S",
                  os.path.join(PKG, "csrc", HAND_SCHEDULED), "-o", asm_path], asm_path))
    if verbose:
        for _, _, cmd, _ in jobs:
            print(" ".join(cmd), flush=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(jobs), 6)) as pool:
        results = list(pool.map(lambda j: run(j[2]), jobs))
    lines, failed = [], []
    for (kind, src, _, _), (rc, out_lines) in zip(jobs, results):
        if kind == "obj":
            lines += out_lines
        if rc != 0:
            failed.append((src, out_lines))
    shown = "\n".join(l for i, l in enumerate(lines) if "packed-fp32-ops" not in l and not is_remark(lines, i))
    if verbose and shown.strip():
        print(shown, flush=True)
    if failed:
        raise RuntimeError("hipcc failed:\n" + "\n".join("\n".join(l for l in o if "packed-fp32-ops" not in l) for _, o in failed))
    if os.path.exists(out):
        os.remove(out)
    spilled = scratch_users(lines)
    if spilled:
        # The SSMM kernels issue their MFMAs (and, the hand-scheduled ones, their loads) as asm the
        # compiler knows nothing about: a spilled accumulator is stored right behind the MFMA that
        # defines it, before the result is written, and a spilled load destination before it has
        # landed.  No such kernel may use scratch memory.
        raise RuntimeError("kernels that must not spill use scratch memory: " + ", ".join(spilled))
    parked = agpr_parkers(lines)
    if parked:
        # Under register pressure the compiler also parks VGPRs in unused accumulation registers
        # (no scratch, so the check above does not see it).
        raise RuntimeError("hand-scheduled kernels with more accumulation registers than accumulators: " + ", ".join(parked))
    found = in_flight_hazards(open(asm_path).read().split("\n"))
    if found:
        # The thing itself: an instruction that reads or writes a register between the asm load that
        # targets it and the wait that covers that load -- a copy, a save to an accumulation register,
        # a spill, a reuse, or an MFMA issued behind a wait that counts wrong.
        for k, n, t, r in found[:20]:
            print(f"{k}: line {n}: {t}   (v{r} in flight)")
        raise RuntimeError(f"{len(found)} accesses to registers of loads in flight in: "
                           + ", ".join(sorted({k for k, _, _, _ in found})))
    objs = [j[3] for j in jobs if j[0] == "obj"]
    rc, link_out = run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out])
    if rc != 0:
        raise RuntimeError("link failed:\n" + "\n".join(link_out))
    return out


def build_probe(verbose=True):
    """The MFMA rate and HBM streaming probes: a library of its own that only bench.py loads."""
    srcs = sorted(glob.glob(os.path.join(PKG, "csrc", "probe", "*.hip")))
    cmd = [hipcc(), *HIPCC_FLAGS, "-shared", "-I", os.path.join(PKG, "csrc", "probe"), *srcs, "-o", PROBE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    rc, out = run(cmd)
    if rc != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in out if "packed-fp32-ops" not in l))
    return PROBE_LIB


def is_remark(lines, i):
    """A resource-usage remark, or one of the two source-echo lines hipcc prints under it."""
    if "-Rpass-analysis=kernel-resource-usage" in lines[i]:
        return True
    return any("remark: Function Name" in lines[j] for j in (i - 1, i - 2) if j >= 0)


def scratch_users(lines):
    """Names of SSMM matrix kernels whose resource report shows scratch memory."""
    bad, name = [], None
    for l in lines:
        if "remark: Function Name:" in l:
            name = l.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in l and name and "ssmm_kernel" in name:
            if int(l.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0:
                bad.append(name)
    return sorted(set(bad))


def accumulator_registers(name):
    """AGPRs the accumulators of an ssmm_kernel2 instance need, from its mangled template arguments
    <GATEUP, VEC, MT, NT, WM, WN, DS, OCC, SPLITK, ANYACT>; None for any other function."""
    m = re.match(r"_ZN4ssmm12ssmm_kernel2I((?:L[bi]\d+E)+)E", name)
    if not m:
        return None
    a = [int(v) for v in re.findall(r"L[bi](\d+)E", m.group(1))]
    if len(a) < 4:
        return None
    gateup, vec, mt, nt = a[:4]
    return min(256, (2 if gateup else 1) * mt * (2 if vec else 1) * nt * 16)


def agpr_parkers(lines, slack=8):
    """Names of hand-scheduled kernels whose resource report shows more AGPRs than their
    accumulators take (plus a few the compiler may use for ordinary values)."""
    bad, name = [], None
    for l in lines:
        if "remark: Function Name:" in l:
            name = l.split("Function Name:")[1].split()[0]
        elif "remark:     AGPRs:" in l and name:
            need = accumulator_registers(name)
            if need is not None and int(l.split("AGPRs:")[1].split()[0]) > need + slack:
                bad.append(name)
    return sorted(set(bad))


# ---------------------------------------------------------------------------------------------
# Registers of asm loads in flight, checked on the device assembly.
#
# Model.  A wave's loads return in order, so a load is complete once `s_waitcnt vmcnt(N)` has been
# passed with at most N loads issued after it.  State at a program point: for every vector register
# that is the destination of an asm load not yet known complete, the least number of loads that can
# have been issued behind that load on any path to the point.  Stores are not counted as "behind"
# (they may retire out of order with loads: not counting them only makes the check stricter).
# Transfer: a load adds one to every entry and enters its own destinations at zero; a wait with
# vmcnt(N) drops the entries that have reached N.  Join of paths: entry-wise minimum.  The state is
# carried over the control-flow graph of the kernel to a fixed point; then every instruction that
# names a register present in its incoming state is a finding.  Only loads written as asm are
# entered (the compiler tracks its own); every load counts as "behind".
# ---------------------------------------------------------------------------------------------
_LOAD = re.compile(r"^(global_load|buffer_load|flat_load|scratch_load|global_atomic\w*\s.*\bglc\b|global_atomic\w*\s.*\bsc0\b)")
_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_BRANCH = re.compile(r"^s_c?branch\w*\s+(\.L\w+)")
_SAT = 64   # counts saturate here (vmcnt holds six bits)


def _vregs(text):
    regs = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


def _vmcnt(text):
    """N of an s_waitcnt that waits on vmcnt, else None."""
    m = re.search(r"vmcnt\((\d+)\)", text)
    if m:
        return int(m.group(1))
    m = re.match(r"s_waitcnt\s+(0x[0-9a-fA-F]+|\d+)\s*$", text)
    if m:   # raw immediate (gfx9: vmcnt = bits 3:0 and 15:14)
        imm = int(m.group(1), 0)
        return (imm & 0xF) | (((imm >> 14) & 0x3) << 4)
    return None


def _kernel_bodies(asm_lines, prefix):
    """(name, [(line number, text, in_asm)]) of every function whose label starts with prefix."""
    cur, body, inasm = None, [], False
    for i, l in enumerate(asm_lines):
        m = re.match(r"^(%s\S*):" % re.escape(prefix), l)
        if m:
            cur, body, inasm = m.group(1), [], False
            continue
        if cur is None:
            continue
        t = l.split(";")[0].strip() if "#ASM" not in l else l.strip()
        if l.startswith(".Lfunc_end") or re.match(r"^[A-Za-z_]\w*:", l):   # the function's end, or the next function
            yield cur, body
            cur = None
            continue
        if "#ASMSTART" in t:
            inasm = True
            continue
        if "#ASMEND" in t:
            inasm = False
            continue
        if not t or t.startswith(("//", ".p2align", ".loc", ".cfi", ".file", ".section", ".type", ".size", ".set", ".amdhsa")):
            continue
        body.append((i + 1, t, inasm))
    if cur is not None:
        yield cur, body


def in_flight_hazards(asm_lines, prefix="_ZN4ssmm12ssmm_kernel2"):
    """[(kernel, line number, text, register)]: instructions that name a register an asm load in flight targets."""
    found = []
    for name, body in _kernel_bodies(asm_lines, prefix):
        # basic blocks
        starts = {0}
        labels = {}
        for k, (_, t, _) in enumerate(body):
            m = re.match(r"^(\.L\w+):", t)
            if m:
                labels[m.group(1)] = k
                starts.add(k)
            if _BRANCH.match(t) or t.startswith(("s_endpgm", "s_setpc")):
                starts.add(k + 1)
        order = sorted(s for s in starts if s < len(body))
        block_of = {s: n for n, s in enumerate(order)}
        ends = order[1:] + [len(body)]
        succ = []
        for s, e in zip(order, ends):
            last = body[e - 1][1]
            out = []
            m = _BRANCH.match(last)
            if m and m.group(1) in labels:
                out.append(block_of[labels[m.group(1)]])
            if not (last.startswith(("s_branch", "s_endpgm", "s_setpc"))) and e < len(body):
                out.append(block_of[e])
            succ.append(out)

        def flow(state, s, e, report):
            st = dict(state)
            for k in range(s, e):
                ln, t, inasm = body[k]
                if re.match(r"^\.L\w+:", t):
                    continue
                regs = _vregs(t)
                is_load = bool(_LOAD.match(t))
                dests = set()
                if is_load and inasm:
                    head = t.split(",")[0]
                    dests = _vregs(head) if not t.startswith("global_load_lds") else set()
                if report is not None:
                    for r in sorted((regs - dests) & st.keys()):
                        report.append((name, ln, t, r))
                    for r in sorted(dests & st.keys()):    # a second load into a register whose first has not landed
                        report.append((name, ln, t, r))
                n = _vmcnt(t) if t.startswith("s_waitcnt") else None
                if n is not None:
                    st = {r: c for r, c in st.items() if c < n}
                if is_load:
                    st = {r: min(c + 1, _SAT) for r, c in st.items()}
                    for r in dests:
                        st[r] = 0
            return st

        entry = [None] * len(order)
        entry[0] = {}
        work = [0]
        while work:
            b = work.pop()
            out = flow(entry[b], order[b], ends[b], None)
            for nb in succ[b]:
                if entry[nb] is None:
                    entry[nb] = dict(out)
                    work.append(nb)
                else:
                    merged = dict(entry[nb])
                    changed = False
                    for r, c in out.items():
                        if r not in merged or c < merged[r]:
                            merged[r] = c
                            changed = True
                    if changed:
                        entry[nb] = merged
                        work.append(nb)
        for b in range(len(order)):
            if entry[b] is not None:
                flow(entry[b], order[b], ends[b], found)
    return found


def audit(verbose=True):
    """The in-flight check alone, on a fresh compile of the hand-scheduled source to assembly."""
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "ssmm_ffn.s")
        rc, lines = run([hipcc(), *HIPCC_FLAGS, *INCLUDES, "--cuda-device-only", "-S",
                         os.path.join(PKG, "csrc", HAND_SCHEDULED), "-o", out])
        if rc != 0:
            raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
        found = in_flight_hazards(open(out).read().split("\n"))
    if verbose:
        for k, n, t, r in found[:20]:
            print(f"{k}: line {n}: {t}   (v{r} in flight)")
        print(f"{len(found)} accesses to registers of loads in flight")
    if found:
        raise RuntimeError("hand-scheduled kernels touch registers of loads in flight")


def build_tuning(verbose=True, extra=()):
    return build(verbose=verbose, extra=["-DSSMM_TUNING", *extra], out=TUNE_LIB)


def build_all(verbose=True, extra=()):
    """The three libraries; the two builds of the SSMM sources run side by side."""
    with concurrent.futures.ThreadPoolExecutor(max_workers=3) as pool:
        jobs = [pool.submit(build, verbose, extra), pool.submit(build_tuning, verbose, extra), pool.submit(build_probe, verbose)]
        return [j.result() for j in jobs]


if __name__ == "__main__":
    if sys.argv[1:] == ["--audit"]:
        audit()
    else:
        build_all(extra=sys.argv[1:])
