"""Static checks of the generated gfx950 instruction stream for the hazards the hand-written assembly must respect.

Parts of the kernels are inline assembly that the compiler does not look into (the score MFMAs of the dK/dV and
forward kernels with architectural destination tuples; exponentials, conversions and packs pinned to their MFMA slots), so the wait states
the compiler would otherwise insert are the author's responsibility.  This module compiles a kernel source to assembly
and verifies, instruction by instruction:

1. MFMA chains (`check_mfma_chains`, for the dK/dV kernel and the forward kernel, whose score MFMAs are assembly;
   elsewhere MFMAs are compiler builtins and the compiler supplies the wait states itself): from the first MFMA that writes an architectural tuple with a fresh C operand to
   the end of its chain (an `s_nop 11`, or the `; chain end` marker), nothing but MFMAs touches the chain's registers
   and no control flow intervenes; after a `; chain end` marker (no wait states by design) no non-MFMA instruction
   touches those registers for the next 16 issue cycles at least.
2. Transcendentals (`check_trans_use`): the instruction directly after a `v_exp_f32` (and its kin) does not read its
   result unless it is itself a transcendental or an `s_nop` (one wait state is required on this architecture).

    python -m paper_2510_18121_amd.isa_check            # compiles csrc/ca_bwd.hip and csrc/ca_fwd.hip, prints findings
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
MFMA = "v_mfma_f32_32x32x16_bf16"
TRANS = ("v_exp_f32", "v_log_f32", "v_rcp_f32", "v_rsq_f32", "v_sqrt_f32", "v_sin_f32", "v_cos_f32")
WINDOW = 16  # issue cycles after a "; chain end" marker in which the chain's registers must stay untouched


def compile_to_asm(source: str) -> str:
    """Device-side assembly of one kernel source, with the flags of the library build."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes", "-Wno-inline-asm",
               "-Wno-int-to-pointer-cast", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
               "-o", out, os.path.join(CSRC, source)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + r.stderr)
        return open(out).read()


def kernel_bodies(asm: str, name_part: str):
    """The instruction streams (label to s_endpgm) of the kernels whose mangled name contains name_part."""
    out, cur = [], None
    for line in asm.split("\n"):
        if cur is None:
            if re.match(r"^_Z\w*" + re.escape(name_part) + r"\w*:", line):
                cur = [line]
        else:
            cur.append(line)
            if line.strip().startswith("s_endpgm"):
                out.append("\n".join(cur))
                cur = None
    return out


def _vregs(text: str) -> set:
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def check_mfma_chains(asm: str):
    """Returns (number of chains, number of '; chain end' markers, list of findings)."""
    first = re.compile(MFMA + r" v\[(\d+):(\d+)\], .*, (0|v\[(\d+):(\d+)\])$")
    any_v = re.compile(MFMA + r" v\[(\d+):(\d+)\]")
    flow = re.compile(r"(s_cbranch|s_branch|\.LBB|s_endpgm)")
    chain = watch = None
    left = n = marks = 0
    bad = []
    for no, line in enumerate(asm.split("\n"), 1):
        t = line.strip()
        if t.startswith("; chain end"):
            if chain is None:
                bad.append((no, "marker without an open chain"))
            watch, left, chain = chain, WINDOW, None
            marks += 1
            continue
        if not t or t.startswith(";"):
            continue
        if watch is not None:
            if flow.match(t):
                bad.append((no, "control flow inside the window after a chain end: " + t))
                watch = None
            else:
                is_mfma = t.startswith("v_mfma")
                if not is_mfma and _vregs(t) & watch:
                    bad.append((no, "chain registers touched inside the window: " + t))
                m = re.match(r"s_nop (\d+)", t)
                left -= int(m.group(1)) + 1 if m else 8 if is_mfma else 1
                if left <= 0:
                    watch = None
        m = first.match(t)
        if m and m.group(3) != "0" and m.group(4) == m.group(1):
            m = None  # accumulating onto itself: a later link, not a first MFMA
        if m:
            if chain is None:
                chain, n = set(), n + 1
            chain |= set(range(int(m.group(1)), int(m.group(2)) + 1))
            continue
        if chain is not None:
            if t.startswith("s_nop 11"):
                chain = None
            elif flow.match(t):
                bad.append((no, "control flow inside a chain: " + t))
                chain = None
            else:
                m2 = any_v.match(t)
                if m2:
                    chain |= set(range(int(m2.group(1)), int(m2.group(2)) + 1))
                elif _vregs(t) & chain:
                    bad.append((no, "chain registers touched before the chain's end: " + t))
    return n, marks, bad


def check_trans_use(asm: str):
    """Returns (number of transcendental instructions, list of findings)."""
    ins = []
    for line in asm.split("\n"):
        t = line.split(";")[0].strip()
        if t and not t.endswith(":") and not t.startswith(".") and not t.startswith("#"):
            ins.append(t)
    n, bad = 0, []
    for a, b in zip(ins, ins[1:]):
        if not a.split()[0].startswith(TRANS):
            continue
        n += 1
        dst = _vregs(a.split(None, 1)[1].split(",")[0])
        op = b.split()[0]
        if op.startswith(TRANS) or op.startswith("s_nop"):
            continue
        parts = b.split(None, 1)
        if len(parts) < 2:
            continue
        ops = parts[1].split(",")
        reads = set()
        for o in (ops if op.startswith(("v_mfma", "ds_write", "global_store")) else ops[1:]):
            reads |= _vregs(o)
        if dst & reads:
            bad.append((a, b))
    return n, bad


def main():
    status = 0
    for src in ("ca_bwd.hip", "ca_fwd.hip"):
        asm = compile_to_asm(src)
        for body in kernel_bodies(asm, "ca_bwd_dkv_kernel") + kernel_bodies(asm, "ca_fwd_kernel"):
            n, marks, bad = check_mfma_chains(body)
            print(f"{src}: {body.split(':')[0]}: {n} hand-written MFMA chains, {marks} chain-end markers, "
                  f"{len(bad)} findings")
            for f in bad:
                print("   line", *f)
            status |= bool(bad)
        bad = []
        nt, badt = check_trans_use(asm)
        print(f"{src}: {nt} transcendental instructions, {len(badt)} findings")
        for f in badt:
            print("  ", *f)
        status |= bool(bad or badt)
    raise SystemExit(status)


if __name__ == "__main__":
    main()
