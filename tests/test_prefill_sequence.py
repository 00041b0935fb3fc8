"""Static checks of the generated instruction sequence of the prompt-chunk kernel (no GPU needed).

The sequence is one inline-asm statement; the compiler only knows about the registers the
statement declares, so every register the sequence names must be one of its operands or
clobbers, and every path through one iteration must meet the workgroup barrier exactly once
(a wave that skipped a barrier would leave the others waiting).
"""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_08671_amd", "csrc")


def test_header_on_disk_matches_generator():
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_prefill_sequence.py"), "--check"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr


def sequence_lines():
    text = open(os.path.join(CSRC, "attn_prefill_sequence.h")).read()
    lines = []
    for l in text.split("\n"):
        m = re.search(r'"(.*?)\\n(\\t)?"', l)
        if not m:
            continue
        head = l.strip().split(" ")[0]
        prefix = {"MFMA": "MFMA", "CVT": "CVT"}.get(head, "")
        lines.append(prefix + m.group(1))
    assert len(lines) > 1000
    return lines


def regs_in(text, kind):
    out = set()
    for a, b in re.findall(rf"\b{kind}\[(\d+):(\d+)\]", text):
        out.update(range(int(a), int(b) + 1))
    out.update(int(a) for a in re.findall(rf"\b{kind}(\d+)\b", text))
    return out


def declared_registers():
    """registers pinned as operands of the asm statement plus the generated clobber list"""
    body = open(os.path.join(CSRC, "attn_prefill_body.h")).read()
    start = body.index("#define FSF_TILE_OPERANDS")
    ops = body[start:body.index("#undef FSF_TILE_OPERANDS")]
    ops = ops[:ops.index("if constexpr")]
    pinned = re.findall(r'\{([vsa][^}]*)\}', ops)
    gen = open(os.path.join(CSRC, "attn_prefill_sequence.h")).read()
    clob = gen[gen.index("#define FSF_TILE_CLOBBERS"):gen.index("#define FSF_TILE_SEQUENCE")]
    pinned += re.findall(r'"([vsa]\d+)"', clob)
    text = " ".join(pinned)
    return regs_in(text, "v"), regs_in(text, "s"), regs_in(text, "a")


def test_sequence_only_touches_declared_registers():
    v_ok, s_ok, a_ok = declared_registers()
    assert len(v_ok) > 200 and len(s_ok) > 30 and len(a_ok) == 256
    for l in sequence_lines():
        if l.endswith(":"):
            continue
        code = re.sub(r"offset:\S+", "", l)
        code = re.sub(r"\.Lfsf_\w+", "", code)
        bad_v = regs_in(code, "v") - v_ok
        bad_s = regs_in(code, "s") - s_ok
        bad_a = regs_in(code, "a") - a_ok
        assert not bad_v and not bad_s and not bad_a, f"{l}: v{sorted(bad_v)} s{sorted(bad_s)} a{sorted(bad_a)} not declared"


def test_every_iteration_has_exactly_one_barrier_on_every_path():
    """Iterations are delimited by the increment of the step counter (s97); between two
    increments there is exactly one s_barrier and it is not inside any skippable region
    (no forward branch jumps over it)."""
    lines = sequence_lines()
    first = next(i for i, l in enumerate(lines) if l.startswith(".Lfsf_g0_"))
    assert sum(l.startswith("s_barrier") for l in lines[:first]) == 1   # the one before QK(0)
    chunks, cur = [], []
    for l in lines[first:]:
        cur.append(l)
        if l.startswith("s_add_u32 s97, s97, 1"):
            chunks.append(cur)
            cur = []
    assert len(chunks) == 4  # two steady and two general iterations
    for ch in chunks:
        idx = [i for i, l in enumerate(ch) if l.startswith("s_barrier")]
        assert len(idx) == 1
        b = idx[0]
        labels = {l[:-1]: i for i, l in enumerate(ch) if l.endswith(":")}
        for i, l in enumerate(ch[:b]):
            m = re.match(r"s_c?branch\w*\s+(\S+)", l)
            if m and m.group(1) in labels:
                assert labels[m.group(1)] < b, f"branch '{l}' can skip the barrier"


def test_lds_offsets_stay_inside_the_four_slots():
    for l in sequence_lines():
        m = re.search(r"offset:(\d+)", l)
        if m:
            off = int(m.group(1))
            if l.startswith("ds_read_b64_tr_b16"):   # V addresses already include the V ring base
                assert off < 32768
            elif l.startswith("ds_read"):
                assert off < 32768                  # K slots
            else:
                assert off < 4096                   # global loads and stores of a row
