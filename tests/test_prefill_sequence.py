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

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_08671_amd", "csrc")


def test_header_on_disk_matches_generator():
    """The header is a build product (not tracked): where a build has left one, it is the generator's output."""
    if not os.path.exists(os.path.join(CSRC, "attn_prefill_sequence.h")):
        pytest.skip("no build has run in this tree yet")
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_prefill_sequence.py"), "--check"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr


def sequence_lines():
    sys.path.insert(0, CSRC)
    try:
        import gen_prefill_sequence
        text = gen_prefill_sequence.render()
    finally:
        sys.path.remove(CSRC)
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


def iteration_chunks():
    lines = sequence_lines()
    first = next(i for i, l in enumerate(lines) if l.startswith(".Lfsf_g0_"))
    chunks, cur = [], []
    for l in lines[first:]:
        cur.append(l)
        if l.startswith("s_add_u32 s97, s97, 1"):
            chunks.append(cur)
            cur = []
    return lines[:first], chunks


def lds_slots(chunk):
    """(K slots read, V slots read, K slots written, V slots written) of an instruction list; LDS is
    K slot 0, K slot 1, V slot 0, V slot 1, 16 KB each; V reads address the V ring through their
    register, copies address LDS through M0 = first copy row of the wave + immediate"""
    kr, vr, kw, vw = set(), set(), set(), set()
    m0 = None
    for l in chunk:
        m = re.match(r"ds_read_b128 .* offset:(\d+)", l)
        if m:
            kr.add(int(m.group(1)) // 16384)
        m = re.match(r"ds_read_b64_tr_b16 .* offset:(\d+)", l)
        if m:
            vr.add(int(m.group(1)) // 16384)
        m = re.match(r"s_add_u32 m0, s81, (\d+)", l)
        if m:
            m0 = int(m.group(1))
        if l.startswith("global_load_lds"):
            assert m0 is not None
            (kw if m0 < 32768 else vw).add((m0 % 32768) // 16384)
            m0 = None   # every copy sets M0 anew
    return kr, vr, kw, vw


def test_lds_slots_alternate_and_copies_never_touch_what_the_iteration_reads():
    """Iteration b (parity s = b & 1) reads K(b+1) and V(b-1) from slots 1-s and copies K(b+2) and
    V(b) into slots s, which the next iteration reads: within an iteration reads and copies
    are disjoint, and the slots swap from one iteration to the next.  The copies all come after
    the iteration's barrier, which directly follows the wait for the wave's own earlier copies."""
    prologue, chunks = iteration_chunks()
    # order of the chunks in the sequence: steady s=0, steady s=1, general s=0, general s=1
    for chunk, s in zip(chunks, (0, 1, 0, 1)):
        kr, vr, kw, vw = lds_slots(chunk)
        assert kr == {1 - s} and vr == {1 - s}, (s, kr, vr)
        assert kw == {s} and vw == {s}, (s, kw, vw)
        b = next(i for i, l in enumerate(chunk) if l.startswith("s_barrier"))
        assert chunk[b - 1].startswith("s_waitcnt vmcnt(0)")
        assert all(not l.startswith("global_load_lds") for l in chunk[:b])
        assert sum(l.startswith("s_waitcnt vmcnt") for l in chunk) == 1   # copies are only waited for at the hand-over
    # before the first iteration: K(0) -> K slot 0, K(1) -> K slot 1, QK(0) reads slot 0 after the barrier
    kr, vr, kw, vw = lds_slots(prologue)
    assert kw == {0, 1} and vw == set() and kr == {0} and vr == set()
    b = next(i for i, l in enumerate(prologue) if l.startswith("s_barrier"))
    assert all(not l.startswith("ds_read") for l in prologue[:b])
    assert all(not l.startswith("global_load_lds") for l in prologue[b:])


def test_waits_cover_every_lds_read_before_its_mfma():
    """Replay the LDS reads and waits of every MFMA block: when an MFMA is issued, the reads that
    filled its fragment registers must be older than the `s_waitcnt lgkmcnt(n)` allowance (LDS
    reads complete in order; scalar loads only make the count more conservative)."""
    lines = sequence_lines()
    outstanding = []          # destination register ranges of reads not yet known to be complete
    for l in lines:
        m = re.match(r"ds_read_\w+ a\[(\d+):(\d+)\]", l)
        if m:
            outstanding.append((int(m.group(1)), int(m.group(2))))
            continue
        m = re.match(r"s_waitcnt (?:vmcnt\(\d+\) )?lgkmcnt\((\d+)\)", l)
        if m:
            n = int(m.group(1))
            outstanding = outstanding[len(outstanding) - n:] if n else []
            continue
        if l.startswith("MFMA"):
            m = re.search(r"MFMA \S+ a\[(\d+):(\d+)\]|MFMA \S+, a\[(\d+):(\d+)\]", l)
            a_lo, a_hi = [int(x) for x in re.findall(r", a\[(\d+):(\d+)\], ", l)[0]]
            for lo, hi in outstanding:
                assert hi < a_lo or lo > a_hi, f"{l}: fragment a[{a_lo}:{a_hi}] may still be in flight"
        if l.endswith(":") or l.startswith("s_cbranch") or l.startswith("s_branch"):
            pass  # blocks are straight-line between their first read and last MFMA
