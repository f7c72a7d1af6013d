"""Static check of the MFMA data hazards around hand-written (inline asm) matrix instructions.

The kernels issue their steady-state MFMAs as volatile asm statements, which the compiler's
hazard recogniser does not see as matrix instructions.  Two rules that it would otherwise
enforce with s_nop are therefore checked here on the generated gfx950 assembly:

  A. a vector-ALU write of a register must be at least 2 wait states old when an MFMA reads
     that register as one of its A/B/C operands;
  B. the result of an 8-pass MFMA (32x32x16 bf16) must be at least 11 wait states old when
     any instruction other than an MFMA touches it (16-pass 32x32x2 f32: 19).

The direct-to-LDS loads (asm as well) take their LDS target from M0, and several of them share
one M0 value set by an asm statement the compiler knows nothing about:

  C. in a function that contains such loads, no instruction outside the asm statements may
     write M0.

Wait states are counted like the compiler does: one per instruction, N+1 for `s_nop N`;
an intervening MFMA counts as its own pass count because it occupies the matrix pipe that
long.  Only hazards with an asm MFMA on one side are reported (compiler-emitted MFMAs are
already covered by the compiler).  The scan is linear per function, which covers the
fall-through order in which the register allocator places its copies.

Run as a module to check the library sources:  python -m paper_2409_04431_amd.isa_check
"""
import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

from .build import CSRC, HIPCC_FLAGS, SOURCES

_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+))")
_PASSES = {"v_mfma_f32_32x32x16_bf16": 8, "v_mfma_f32_32x32x2_f32": 16, "v_mfma_f32_32x32x2f32": 16}
_AFTER_MFMA = {8: 11, 16: 19}


def _regs(operand):
    """Set of ('v'|'a', index) named by one operand string."""
    out = set()
    for m in _REG.finditer(operand):
        kind = m.group(1)
        if m.group(4) is not None:
            out.add((kind, int(m.group(4))))
        else:
            out.update((kind, i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
    return out


class Inst:
    __slots__ = ("op", "dst", "src", "in_asm", "text", "line")

    def __init__(self, text, in_asm, line):
        self.text, self.in_asm, self.line = text, in_asm, line
        parts = text.split(None, 1)
        self.op = parts[0]
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        writes_first = self.op.startswith(("v_", "ds_read", "global_load", "buffer_load", "scratch_load")) \
            and not self.op.startswith(("v_cmp", "v_cmpx", "global_load_lds"))
        self.dst = _regs(ops[0]) if (ops and writes_first) else set()
        self.src = set()
        for o in (ops[1:] if writes_first else ops):
            self.src |= _regs(o)

    @property
    def is_mfma(self):
        return self.op.startswith("v_mfma")

    @property
    def is_valu(self):
        return self.op.startswith("v_") and not self.is_mfma

    def wait_states(self):
        if self.op == "s_nop":
            return int(self.text.split()[1], 0) + 1
        if self.is_mfma:
            return _PASSES.get(self.op, 4)
        return 1


def parse_functions(asm_text):
    """Yield (name, [Inst]) for every function of an AMDGPU assembly listing."""
    name, insts, in_asm = None, [], False
    for ln, raw in enumerate(asm_text.splitlines(), 1):
        line = raw.strip()
        if line.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if line.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not line or line.startswith((";", ".", "//")):
            continue
        m = re.match(r"^([A-Za-z_][\w$.]*):", line)
        if m:
            if not line.startswith(".L"):
                if name and insts:
                    yield name, insts
                name, insts = m.group(1), []
            continue
        code = line.split(";")[0].strip()
        if not code or name is None:
            continue
        if code.startswith("s_endpgm"):
            if insts:
                yield name, insts
            name, insts = None, []
            continue
        insts.append(Inst(code, in_asm, ln))
    if name and insts:
        yield name, insts


def check_function(insts):
    """Return a list of (rule, message) violations."""
    bad = []
    for i, ins in enumerate(insts):
        if not ins.is_mfma:
            continue
        # Rule A: look back
        if ins.in_asm:
            ws, j = 0, i - 1
            while j >= 0 and ws < 2:
                p = insts[j]
                if p.is_valu and (p.dst & ins.src):
                    bad.append(("A", f"line {p.line}: '{p.text}' feeds '{ins.text}' (line {ins.line}) after {ws} wait states"))
                    break
                ws += p.wait_states()
                j -= 1
        # Rule B: look ahead
        if ins.in_asm:
            need = _AFTER_MFMA[_PASSES.get(ins.op, 8)]
            ws, j = 0, i + 1
            while j < len(insts) and ws < need:
                n = insts[j]
                if not n.is_mfma and ((n.src | n.dst) & ins.dst):
                    bad.append(("B", f"line {n.line}: '{n.text}' touches the result of '{ins.text}' (line {ins.line}) after {ws} wait states"))
                    break
                if n.is_mfma and (n.dst & ins.dst) and n.dst != ins.dst:
                    bad.append(("B", f"line {n.line}: '{n.text}' partly overlaps the result of '{ins.text}' (line {ins.line})"))
                    break
                ws += n.wait_states()
                j += 1
    # Rule C
    if any(i.in_asm and i.op.startswith("global_load_lds") for i in insts):
        for ins in insts:
            if not ins.in_asm and re.match(r"^s_\w+\s+m0\b", ins.text):
                bad.append(("C", f"line {ins.line}: '{ins.text}' writes M0 outside the asm statements"))
    return bad


def check_text(asm_text):
    out = []
    for name, insts in parse_functions(asm_text):
        for rule, msg in check_function(insts):
            out.append(f"{name}: rule {rule}: {msg}")
    return out


def compile_to_asm(extra_flags=()):
    """Device-only assembly of the library sources with the product's flags."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    with tempfile.TemporaryDirectory() as td:
        def one(s):
            out = os.path.join(td, s + ".s")
            cmd = [hipcc] + flags + list(extra_flags) + ["--cuda-device-only", "-S", "-o", out, os.path.join(CSRC, s)]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + res.stderr)
            with open(out) as f:
                return f.read()
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 16)) as pool:
            texts = list(pool.map(one, SOURCES))
    return "\n".join(texts)


if __name__ == "__main__":
    problems = check_text(compile_to_asm())
    for p in problems:
        print(p)
    print(f"{len(problems)} hazard(s)")
    sys.exit(1 if problems else 0)
