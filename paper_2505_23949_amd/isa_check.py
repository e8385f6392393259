"""Static check of the compiled kernels for hazards around hand-written instructions.

A few operations of the kernels are written as bare instructions (inline assembly) so that they stay the one
instruction meant.  The compiler treats such a statement as opaque when it inserts the wait states that gfx950
needs between certain pairs of instructions, so two kinds of hazard can slip through, and both give wrong
numbers silently:

  H1  the result of a transcendental instruction (v_rcp, v_exp, ...) read by the vector instruction issued
      right behind it (one wait state needed);
  H2  a DPP instruction reading a register that a vector instruction wrote fewer than two wait states earlier.

`hazards()` scans an ISA listing for both, with a hand-written instruction on the reading side (H1) or the
writing side (H2).  Hand-written instructions are recognised by how they are printed: without the encoding suffix
the compiler gives its own 32-bit ones (`v_min_f32` against `v_min_f32_e32`), or as the one form written with it
(`v_mul_f32_e64 ... clamp`).  The 64-bit minimum and maximum print without a suffix whoever wrote them; all of
them are treated as hand-written, which only makes the check stricter.  `listing()` compiles one translation
unit to such a listing.
"""
from __future__ import annotations

import re
import subprocess
import tempfile
from pathlib import Path

from . import build as _build

_TRANS = re.compile(r"^v_(rcp|rcp_iflag|rsq|sqrt|exp|log|sin|cos)_(f16|f32|f64)")
_BARE = ("v_max_f32", "v_min_f32", "v_max_f64", "v_min_f64")


def _regs(token: str) -> set[int]:
    token = token.strip().lstrip("-|").rstrip("|")
    m = re.match(r"^v(\d+)$", token)
    if m:
        return {int(m.group(1))}
    m = re.match(r"^v\[(\d+):(\d+)\]$", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def _hand_written(op: str, rest: str) -> bool:
    return op in _BARE or (op == "v_mul_f32_e64" and rest.rstrip().endswith("clamp"))


def hazards(text: str, name: str = "") -> list[str]:
    """The hazards of kinds H1 and H2 found in an ISA listing, one line of description each."""
    found = []
    recent: list[tuple[str, set[int], int, bool]] = []   # (opcode, registers written, wait states after it, hand-written)
    for number, line in enumerate(text.split("\n"), 1):
        if not line.startswith("\t") or line.strip().startswith((".", ";")):
            if re.match(r"^\S+:", line):
                recent = []          # a label: what ran before is not known
            continue
        body = line.split(";")[0].strip()
        if not body:
            continue
        op, _, rest = body.partition(" ")
        if op == "s_nop":
            extra = int(rest.strip()) + 1
            recent = [(o, d, w + extra, h) for (o, d, w, h) in recent]
            continue
        operands = re.split(r",\s*", re.split(r" (row_|quad_perm|clamp|wave_|bound_ctrl)", rest)[0]) if rest else []
        writes = _regs(operands[0]) if operands and op.startswith("v_") else set()
        reads = set().union(*[_regs(t) for t in operands[1:]]) if len(operands) > 1 else set()
        mine = _hand_written(op, rest)
        if mine and recent:
            o, d, w, _ = recent[-1]
            if _TRANS.match(o) and (d & reads) and w == 0:
                found.append(f"H1 {name}:{number}: `{body}` reads the result of {o} issued right before it")
        if "_dpp" in op or " row_" in rest or "quad_perm" in rest:
            for k, (o, d, w, h) in enumerate(reversed(recent)):
                if k + w >= 2:
                    break
                if h and (d & reads):
                    found.append(f"H2 {name}:{number}: `{body}` reads what {o} wrote {k + w} wait state(s) earlier")
        recent = (recent + [(op, writes, 0, mine)])[-4:]
    return found


def listing(source: Path) -> str:
    """ISA listing of the device code of one translation unit, compiled with the flags of the library."""
    with tempfile.TemporaryDirectory() as tmp:
        out = Path(tmp) / (Path(source).stem + ".s")
        subprocess.run([_build.HIPCC, *_build.FLAGS, "--cuda-device-only", "-S", "-o", str(out), str(source)],
                       check=True, stderr=subprocess.DEVNULL)
        return out.read_text()


def check_all(jobs: int = 6) -> list[str]:
    """Hazards in every translation unit of the library."""
    from concurrent.futures import ThreadPoolExecutor

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        texts = list(pool.map(listing, _build.SOURCES))
    return [h for src, text in zip(_build.SOURCES, texts) for h in hazards(text, Path(src).name)]


if __name__ == "__main__":
    problems = check_all()
    print("\n".join(problems) if problems else "no hazards around hand-written instructions")
    raise SystemExit(1 if problems else 0)
