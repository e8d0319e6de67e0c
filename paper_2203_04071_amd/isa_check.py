#!/usr/bin/env python3
"""Static check of the compiled derived-table kernels (build-time safety net, run by the CPU test suite).

Their inner loops issue LDS reads and global loads from inline assembly and consume the results in LATER asm statements,
after an explicit s_waitcnt.  The compiler believes such a register is valid as soon as the issuing statement ends; if it
ever copied or spilled one in between, it would move stale data (a silent wrong result that depends on register
allocation).  This script scans the generated gfx950 assembly of every instantiation: between the issue of such a load
and the wait that covers it, no instruction may touch the destination registers.  Linear scan per function; two queues
model the in-order retirement of lgkmcnt / vmcnt; loads issued behind a scalar branch inside an asm statement count as
issued only while the loop goes on (they are dropped at a backward branch).

  python -m paper_2203_04071_amd.isa_check            compiles the translation units that hold hand-scheduled kernels to assembly and checks them
  python -m paper_2203_04071_amd.isa_check file.s     checks an existing assembly file
"""
import os
import re
import subprocess
import sys
import tempfile

class RS(set):
    cond = False

def regs(tok):
    out = set()
    for m in re.finditer(r'v\[(\d+):(\d+)\]', tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    tok2 = re.sub(r'v\[\d+:\d+\]', '', tok)
    for m in re.finditer(r'\bv(\d+)\b', tok2):
        out.add(int(m.group(1)))
    return out

def check(path, pattern):
    txt = open(path).read().split('\n')
    fn = None; bad = 0; nfn = 0
    in_asm = False
    lq, vq = [], []      # queues of register sets (oldest first)
    labels = set(); cond = False   # cond: inside an asm block after a forward scalar branch (conditionally issued)
    for ln, line in enumerate(txt, 1):
        s = line.strip()
        m = re.match(r'^(_Z\w+):', line)
        if m:
            fn = m.group(1) if re.search(pattern, m.group(1)) else None
            lq, vq = [], []; in_asm = False; labels = set(); cond = False
            if fn: nfn += 1
            continue
        if fn and re.match(r'^[.\w$]+:', s):
            labels.add(s.split(':')[0]); cond = False; continue
        if fn is None or not s or s.startswith(('.', ';')) and 'ASM' not in s:
            if fn and s.startswith(';;#ASMSTART'): in_asm = True
            if fn and s.startswith(';;#ASMEND'): in_asm = False
            continue
        if s.startswith(';;#ASMSTART'): in_asm = True; cond = False; continue
        if s.startswith(';;#ASMEND'): in_asm = False; cond = False; continue
        if s.startswith('s_endpgm'):
            fn = None; continue
        code = s.split(';')[0].strip()
        if not code: continue
        if code.endswith(':'):
            labels.add(code[:-1]); cond = False; continue
        op = code.split()[0]
        args = code[len(op):]
        if op.startswith('s_cbranch') or op == 's_branch':
            tgt = args.strip()
            if in_asm: cond = True
            elif tgt in labels:      # loop back-edge: what was issued only "if the loop goes on" is absent on the exit path
                lq = [e for e in lq if not getattr(e, 'cond', False)]
                vq = [e for e in vq if not getattr(e, 'cond', False)]
            continue
        if op == 's_waitcnt':
            m1 = re.search(r'lgkmcnt\((\d+)\)', args); m2 = re.search(r'vmcnt\((\d+)\)', args)
            if not m1 and not m2:
                imm = int(args.strip(), 0)
                vm = imm & 0xf | ((imm >> 14) & 3) << 4; lg = (imm >> 8) & 0xf
                if lg < 15: lq = lq[len(lq) - lg:] if lg else []
                if vm < 63: vq = vq[len(vq) - vm:] if vm else []
            else:
                if m1:
                    n = int(m1.group(1)); lq = lq[len(lq) - n:] if n else []
                if m2:
                    n = int(m2.group(1)); vq = vq[len(vq) - n:] if n else []
            continue
        inflight = set().union(*lq, *vq) if (lq or vq) else set()
        used = regs(args)
        if op.startswith('ds_read') or op.startswith('ds_load'):
            dst = regs(args.split(',')[0])
            if (used - dst) & inflight or (not in_asm and dst & inflight):
                print(f"{fn}: line {ln}: {code}  touches in-flight {sorted(used & inflight)}"); bad += 1
            e = RS(dst if in_asm else ()); e.cond = cond; lq.append(e)
            continue
        if op.startswith('ds_') or op.startswith('s_load') or op.startswith('s_buffer_load'):
            if used & inflight:
                print(f"{fn}: line {ln}: {code}  touches in-flight {sorted(used & inflight)}"); bad += 1
            lq.append(set()); continue
        if op.startswith('global_load_lds'):
            e = RS(); e.cond = cond; vq.append(e); continue
        if op.startswith(('global_load', 'scratch_load', 'buffer_load', 'flat_load')):
            dst = regs(args.split(',')[0])
            if (used - dst) & inflight or (not in_asm and dst & inflight):
                print(f"{fn}: line {ln}: {code}  touches in-flight {sorted(used & inflight)}"); bad += 1
            e = RS(dst if in_asm else ()); e.cond = cond; vq.append(e)
            continue
        if op.startswith(('global_store', 'scratch_store', 'buffer_store', 'flat_store', 'global_atomic')):
            if used & inflight:
                print(f"{fn}: line {ln}: {code}  touches in-flight {sorted(used & inflight)}"); bad += 1
            vq.append(set()); continue
        if used & inflight:
            print(f"{fn}: line {ln}: {code}  touches in-flight {sorted(used & inflight)}"); bad += 1
    print(f"checked {nfn} functions, {bad} violations")
    return bad

def compile_to_asm(source, out_path):
    from .build import HIPCC_FLAGS
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + ["-S", "--cuda-device-only", "-o", out_path, source]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed:\n" + r.stdout + r.stderr)


def check_build(pattern='lut_lines_(fast_|wide_)?kernel|lut_grouped_tiled_kernel'):
    """Number of violations in a fresh compilation of the library's device code."""
    from .build import HAND_SCHEDULED
    bad = 0
    with tempfile.TemporaryDirectory() as d:
        for i, source in enumerate(HAND_SCHEDULED):
            path = os.path.join(d, "tu%d.s" % i)
            compile_to_asm(source, path)
            bad += check(path, pattern)
    return bad


if __name__ == '__main__':
    if len(sys.argv) > 1:
        sys.exit(1 if check(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else 'lut_lines_fast_kernel') else 0)
    sys.exit(1 if check_build() else 0)
