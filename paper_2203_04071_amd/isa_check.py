#!/usr/bin/env python3
"""Static check of the compiled derived-table kernels (build-time safety net, run by the CPU test suite).

Their inner loops issue LDS reads and global loads from inline assembly and consume the results in LATER asm statements,
after an explicit s_waitcnt.  The compiler believes such a register is valid as soon as the issuing statement ends; if it
ever copied or spilled one in between, it would move stale data (a silent wrong result that depends on register
allocation).  This script scans the generated gfx950 assembly of every instantiation: between the issue of such a load
and the wait that covers it, no instruction may touch the destination registers.  Every path of a function's
control-flow graph is walked (the compiler rotates loops, so the order of the text is not the order of execution); two
queues model the in-order retirement of lgkmcnt / vmcnt.  The same walk checks that no compiler-generated instruction
touches the accumulators of matrix instructions issued from asm before the kernel has drained the matrix pipe.

  python -m paper_2203_04071_amd.isa_check            compiles the translation units that hold hand-scheduled kernels to assembly and checks them
  python -m paper_2203_04071_amd.isa_check file.s     checks an existing assembly file
"""
import os
import re
import subprocess
import sys
import tempfile

def regs(tok):
    out = set()
    for m in re.finditer(r'v\[(\d+):(\d+)\]', tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    tok2 = re.sub(r'v\[\d+:\d+\]', '', tok)
    for m in re.finditer(r'\bv(\d+)\b', tok2):
        out.add(int(m.group(1)))
    return out


def _trim(q, cap):
    """Oldest entries that name no register cannot matter any more; neither can entries beyond the counter's range."""
    q = list(q)
    while q and not q[0]:
        q.pop(0)
    return tuple(q[-cap:])


def _functions(txt, pattern):
    """(name, [(line number, stripped text)]) of every function whose mangled name matches the pattern."""
    name, body = None, []
    for ln, line in enumerate(txt, 1):
        m = re.match(r'^(_Z\w+):', line)
        if m:
            if name:
                yield name, body
            name = m.group(1) if re.search(pattern, m.group(1)) else None
            body = []
            continue
        if name is None:
            continue
        s = line.strip()
        if s.startswith('.Lfunc_end'):          # (blocks may follow an s_endpgm: the function ends at its end label)
            yield name, body
            name, body = None, []
            continue
        body.append((ln, s))
    if name:
        yield name, body


def _merge(q1, q2):
    """Both queues end with their newest entry; a wait keeps the newest n.  Entry-wise union, aligned at that end."""
    if len(q1) < len(q2):
        q1, q2 = q2, q1
    pad = len(q1) - len(q2)
    return tuple(q1[i] | (q2[i - pad] if i >= pad else frozenset()) for i in range(len(q1)))


def _check_function(fn, body, report):
    """Forward data-flow over the function's basic blocks.  State: the queue of LDS / scalar loads and the queue of vector
    memory operations in flight (destination registers of those issued from asm), and the accumulators of matrix
    instructions issued from asm that have not been drained.  Where paths meet, the states are merged entry by entry
    (what MAY be in flight), so the check errs on the side of reporting."""
    prog, labels = [], {}
    for ln, s in body:
        if s.startswith(';;#ASMSTART'):
            prog.append((ln, 'asm+', '', '')); continue
        if s.startswith(';;#ASMEND'):
            prog.append((ln, 'asm-', '', '')); continue
        if not s or s.startswith((';', '.')) and not re.match(r'^[.\w$]+:', s):
            continue
        code = s.split(';')[0].strip()
        if not code:
            continue
        if re.match(r'^[.\w$]+:$', code):
            labels[code[:-1]] = len(prog); continue
        op = code.split()[0]
        prog.append((ln, 'i', op, code[len(op):]))
    state_in_points = set(labels.values())       # where blocks begin
    state_in = {0: ((), (), frozenset())}
    work = [0]
    while work:
        pc = work.pop()
        lq, vq, mf = state_in[pc]
        in_asm = False

        def flow(to):
            old = state_in.get(to)
            new = (lq, vq, mf) if old is None else (_merge(old[0], lq), _merge(old[1], vq), old[2] | mf)
            if new != old:
                state_in[to] = new
                work.append(to)

        first = True
        while pc < len(prog):
            if not first and pc in state_in_points:
                flow(pc)          # fall through into a block that other paths enter as well
                break
            first = False
            ln, kind, op, args = prog[pc]
            pc += 1
            if kind == 'asm+':
                in_asm = True; continue
            if kind == 'asm-':
                in_asm = False; continue
            code = op + args
            if op == 's_endpgm':
                break
            if op.startswith('s_cbranch') or op == 's_branch':
                tgt = args.strip()
                if tgt in labels:
                    flow(labels[tgt])
                    if op == 's_branch':
                        break
                continue
            if op == 's_waitcnt':
                m1 = re.search(r'lgkmcnt\((\d+)\)', args); m2 = re.search(r'vmcnt\((\d+)\)', args)
                if not m1 and not m2:
                    imm = int(args.strip(), 0)
                    vm = imm & 0xf | ((imm >> 14) & 3) << 4; lg = (imm >> 8) & 0xf
                    if lg < 15: lq = lq[len(lq) - lg:] if lg else ()
                    if vm < 63: vq = vq[len(vq) - vm:] if vm else ()
                else:
                    if m1:
                        n = int(m1.group(1)); lq = lq[len(lq) - n:] if n else ()
                    if m2:
                        n = int(m2.group(1)); vq = vq[len(vq) - n:] if n else ()
                continue
            inflight = set().union(*lq, *vq) if (lq or vq) else set()
            used = regs(args)
            # Matrix instructions issued from asm: the compiler does not know that their results need wait states before a
            # vector instruction may read them, so until the kernel drains the pipe (s_nop 15 inside an asm statement) no
            # instruction outside asm may touch an accumulator.
            if op.startswith('v_mfma') and in_asm:
                mf = mf | frozenset(regs(args.split(',')[0]))
            elif op == 's_nop' and in_asm and args.strip() == '15':
                mf = frozenset()
            elif not in_asm and used & mf:
                report(fn, ln, code, f"touches matrix accumulators {sorted(used & mf)} before the pipe is drained")
            if op.startswith('ds_read') or op.startswith('ds_load'):
                dst = regs(args.split(',')[0])
                if (used - dst) & inflight or (not in_asm and dst & inflight):
                    report(fn, ln, code, f"touches in-flight {sorted(used & inflight)}")
                lq = _trim(lq + (frozenset(dst if in_asm else ()),), 15)
                continue
            if op.startswith('ds_') or op.startswith('s_load') or op.startswith('s_buffer_load'):
                if used & inflight:
                    report(fn, ln, code, f"touches in-flight {sorted(used & inflight)}")
                lq = _trim(lq + (frozenset(),), 15); continue
            if op.startswith('global_load_lds'):
                vq = _trim(vq + (frozenset(),), 63); continue
            if op.startswith(('global_load', 'scratch_load', 'buffer_load', 'flat_load')):
                dst = regs(args.split(',')[0])
                if (used - dst) & inflight or (not in_asm and dst & inflight):
                    report(fn, ln, code, f"touches in-flight {sorted(used & inflight)}")
                vq = _trim(vq + (frozenset(dst if in_asm else ()),), 63)
                continue
            if op.startswith(('global_store', 'scratch_store', 'buffer_store', 'flat_store', 'global_atomic')):
                if used & inflight:
                    report(fn, ln, code, f"touches in-flight {sorted(used & inflight)}")
                vq = _trim(vq + (frozenset(),), 63); continue
            if used & inflight:
                report(fn, ln, code, f"touches in-flight {sorted(used & inflight)}")


def check(path, pattern):
    txt = open(path).read().split('\n')
    found = {}
    def report(fn, ln, code, what):
        found.setdefault((fn, ln), f"{fn}: line {ln}: {code}  {what}")
    nfn = 0
    for fn, body in _functions(txt, pattern):
        nfn += 1
        _check_function(fn, body, report)
    for k in sorted(found):
        print(found[k])
    print(f"checked {nfn} functions, {len(found)} violations")
    return len(found)

# ---- the older scan, in the order of the text, for the kernels whose loops the compiler lays out in that order: two
# queues as above; loads issued behind a scalar branch inside an asm statement count as issued only while the loop goes
# on (they are dropped at a backward branch)
class RS(set):
    cond = False

def _regs_unused(tok):
    out = set()
    for m in re.finditer(r'v\[(\d+):(\d+)\]', tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    tok2 = re.sub(r'v\[\d+:\d+\]', '', tok)
    for m in re.finditer(r'\bv(\d+)\b', tok2):
        out.add(int(m.group(1)))
    return out

def check_linear(path, pattern):
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


def check_build(pattern='lut_lines_(fast_)?kernel|lut_grouped_tiled_kernel', graph_pattern='lut_quad_kernel'):
    """Number of violations in a fresh compilation of the library's device code (`pattern`: kernels scanned in text
    order; `graph_pattern`: kernels walked along their control-flow graph)."""
    from .build import HAND_SCHEDULED
    bad = 0
    with tempfile.TemporaryDirectory() as d:
        for i, source in enumerate(HAND_SCHEDULED):
            path = os.path.join(d, "tu%d.s" % i)
            compile_to_asm(source, path)
            bad += check_linear(path, pattern) + check(path, graph_pattern)
    return bad


if __name__ == '__main__':
    if len(sys.argv) > 1:
        sys.exit(1 if check(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else 'lut_lines_fast_kernel') else 0)
    sys.exit(1 if check_build() else 0)
