#!/usr/bin/env python3
"""Writes attn_prefill_sequence.h: the fixed gfx950 instruction sequence a wave runs to walk
one prompt-chunk tile over its 64-key steps (macro FSF_TILE_SEQUENCE, used by
attn_prefill_body.h, which documents the algorithm, the LDS layout and the register map).

    python gen_prefill_sequence.py            # rewrites the header next to this file
    python gen_prefill_sequence.py --check    # exit 1 if the header on disk is out of date

The sequence is emitted as the string of one inline-asm statement.  Two tokens stay macro
parameters so that one sequence serves both element types: MFMA (the 32x32x16 matrix
instruction) and CVT (the packing float -> 2-byte conversion).

A wave owns 64 rows as two 32-row blocks (rb = 0, 1) and runs alone on its SIMD with all 512
registers: 256 vector registers (v) for everything the vector ALU touches and 256 accumulation
registers (a) for what only the matrix core touches.
"""
import os
import sys

# ---- vector registers
V_TMP_COPY = (28, 29)           # temporaries of a clamped copy
V_RHI = [30, 32]                # last visible key of the lane's row in row block rb, minus 4*hg
V_RLO = [31, 33]                # first visible key ..., minus 4*hg
V_RHI_REL, V_RLO_REL = 34, 35   # the same relative to the first key of the step
VOFF = [36, 37, 38, 39]         # lane offsets of the wave's four V copy instructions
KOFF = [40, 41, 42, 43]         # ... of its four K copy instructions
V_M = ['v44', 'v47']            # running reference (log2 domain) per row block
V_L = ['v45', 'v48']            # running sum
V_C = ['v46', 'v49']            # factor of the last raise of the reference
V_SL2, V_NINF = 'v50', 'v51'    # scale*log2(e), -inf
VA = 52                         # v52..v55: LDS address of the lane's V^T fragment, per 32-wide d tile
KA = 56                         # v56..v63: LDS address of the lane's K fragment, per k-step
SB = [64, 128]                  # two S^T buffers of 64 registers: 32*rb + 16*kt + r
PB = 192                        # P^T, 32 registers: 16*rb + r
V_OUT = [224, 226]              # 64-bit address of the lane's output row per row block (+ 8*hg bytes)
V_Q = [228, 230]                # 64-bit address of the lane's query row (+ 16*hg bytes); prologue only
TMP = 232                       # v232..v255: temporaries
# ---- accumulation registers
AO = 0                          # a0..a127: O^T, 64*rb + 16*mt + r
AQ = 128                        # a128..a191: Q^T fragments, 32*rb + 4*t + r
AF, NSLOT = 192, 16             # a192..a255: sixteen 4-register K / V^T fragments in flight
# ---- scalar registers
S_PARTIAL = 's51'               # 0: store normalised outputs; 1: store the unnormalised partial result
S_VBASE = 's[52:53]'            # temporary: address of the V tile being copied
S_RAISED = ['s[88:89]', 's[54:55]']   # lanes whose reference the last softmax raised, per row block
S_LIVE = ['s[56:57]', 's[58:59]']     # lanes whose row exists, per row block
S_NSTEPS, S_JFIRST, S_JLAST = 's60', 's61', 's62'
S_NOMASK_LO, S_NOMASK_HI = 's63', 's64'
S_FAST_LO, S_FAST_HI, S_WHOLE_HI = 's65', 's66', 's67'
S_LAST_ROW, S_KEY_BEGIN, S_WINDOW, S_STEP0 = 's68', 's69', 's70', 's71'
S_SPB_MASK, S_SPB_SHIFT = 's72', 's73'
S_BT, S_KHEAD, S_VHEAD = 74, 76, 78      # 64-bit pairs
S_BLK_BYTES, S_LDS_ROW0 = 's80', 's81'
S_OFF0, S_OFF1 = 's[90:91]', 's[98:99]'  # byte offset of the tiles of step b, of step b+1
S_PHYS, S_PAIRS, S_B = 's94', 's95', 's97'   # physical block of step b+2; steady pairs left; b
# s82..s87, s92, s93, s96: temporaries (s[84:85] offset of step b+2, s[86:87] address of a K tile)

TILE_BYTES = 16384          # one K or V tile in LDS
V_RING = 2 * TILE_BYTES     # K slots at 0 and 16384, V slots at 32768 and 49152
MFMA_DRAIN = ['s_nop 7', 's_nop 3']   # idle cycles before other code may read the last MFMA's result
LOOKAHEAD = 7               # fragments whose LDS reads are in flight ahead of the MFMAs
WAIT_EVERY = 2              # one s_waitcnt per this many fragments

_uid = [0]


def label(name):
    _uid[0] += 1
    return f'.Lfsf_{name}{_uid[0]}_%='


def S(buf, rb, j):
    return f'v{SB[buf] + 32 * rb + j}'


def s_acc(buf, rb, kt):
    b = SB[buf] + 32 * rb + 16 * kt
    return f'v[{b}:{b + 15}]'


def o_acc(rb, mt):
    b = AO + 64 * rb + 16 * mt
    return f'a[{b}:{b + 15}]'


def q_frag(rb, t):
    b = AQ + 32 * rb + 4 * t
    return f'a[{b}:{b + 3}]'


def p_frag(rb, u):
    b = PB + 16 * rb + 4 * u
    return f'v[{b}:{b + 3}]'


# ---------------------------------------------------------------------------------------
def softmax(buf):
    """Online softmax of S^T buffer `buf` (already masked where needed), both row blocks.
    A lane holds 32 scores of one row per row block; the other half-wave holds the row's other
    32.  The scores are replaced in place by the probabilities (fp32); returns (that sequence,
    the conversions that pack them into P^T: register r = pack(p[2r], p[2r+1]))."""
    streams = []   # per row block: groups of instructions that stay together
    for rb in range(2):
        t = [TMP + 12 * rb + i for i in range(4)]
        sa, sb = TMP + 12 * rb + 4, TMP + 12 * rb + 5
        m, l, c = V_M[rb], V_L[rb], V_C[rb]
        s = lambda j: S(buf, rb, j)
        G = [[f'v_max3_f32 v{t[k]}, {s(3 * k)}, {s(3 * k + 1)}, {s(3 * k + 2)}' for k in range(4)]]
        chain = []
        j, k = 12, 0
        while j + 1 < 32:
            chain.append(f'v_max3_f32 v{t[k]}, v{t[k]}, {s(j)}, {s(j + 1)}')
            j += 2
            k = (k + 1) % 4
        G += [chain[0:4], chain[4:8], chain[8:10]]
        G += [[f'v_max3_f32 v{t[0]}, v{t[0]}, v{t[1]}, v{t[2]}'],
              [f'v_max_f32 v{t[0]}, v{t[0]}, v{t[3]}'],
              # the other half-wave holds the other 32 keys of the same rows
              [f'v_mov_b32 v{t[1]}, v{t[0]}', 's_nop 1', f'v_permlane32_swap_b32 v{t[1]}, v{t[0]}'],
              [f'v_max_f32 v{t[0]}, v{t[0]}, v{t[1]}'],
              # raise the running reference only where the maximum outgrew it by more than 2^8
              [f'v_mul_f32 v{t[0]}, {V_SL2}, v{t[0]}'],
              [f'v_max_f32 v{t[1]}, v{t[0]}, {m}'],
              [f'v_sub_f32 v{t[2]}, v{t[1]}, {m}'],
              [f'v_cmp_lt_f32 vcc, 0x41000000, v{t[2]}', f'v_cndmask_b32 v{t[1]}, {m}, v{t[1]}, vcc',
               f's_mov_b64 {S_RAISED[rb]}, vcc'],
              [f'v_sub_f32 v{t[2]}, {m}, v{t[1]}'],
              [f'v_exp_f32 {c}, v{t[2]}', f'v_mov_b32 {m}, v{t[1]}', f'v_mov_b32 v{sa}, 0', f'v_mov_b32 v{sb}, 0'],
              [f'v_mul_f32 {l}, {l}, {c}']]
        # exponent, exponential and sum of element j run one behind the other, so that the
        # slow exponentials are spread evenly through the stream (a run of them keeps the MFMA
        # that is due next from being issued in time)
        for i in range(32 + 2):
            grp = []
            if i < 32:
                grp.append(f'v_fma_f32 {s(i)}, {s(i)}, {V_SL2}, -{m}')
            if 0 <= i - 1 < 32:
                grp.append(f'v_exp_f32 {s(i - 1)}, {s(i - 1)}')
            if 0 <= i - 2 < 32:
                acc_ = sa if (i - 2) % 2 == 0 else sb
                grp.append(f'v_add_f32 v{acc_}, v{acc_}, {s(i - 2)}')
            G.append(grp)
        G += [[f'v_add_f32 v{sa}, v{sa}, v{sb}'], [f'v_add_f32 {l}, {l}, v{sa}']]
        streams.append(G)
    # the two row blocks are independent: alternate their groups, which keeps an instruction
    # away from the one that needs its result
    probs = []
    for ga, gb in zip(*streams):
        probs += ga + gb
    pack = [f'CVT v{PB + 16 * rb + r}, {S(buf, rb, 2 * r)}, {S(buf, rb, 2 * r + 1)}'
            for rb in range(2) for r in range(16)]
    return probs, pack


def pv_program(vslot):
    """O^T += V^T P^T: fragment (u, mt) = keys 16u..16u+15 x d tile mt, shared by both row blocks"""
    prog = []
    for u in range(4):
        for mt in range(4):
            reads = [f'ds_read_b64_tr_b16 a[{{r0}}:{{r1}}], v{VA + mt} offset:{vslot * TILE_BYTES + 16 * u * 256}',
                     f'ds_read_b64_tr_b16 a[{{r2}}:{{r3}}], v{VA + mt} offset:{vslot * TILE_BYTES + (16 * u + 8) * 256}']
            mfmas = [f'MFMA {o_acc(rb, mt)}, a[{{r0}}:{{r3}}], {p_frag(rb, u)}, {o_acc(rb, mt)}' for rb in range(2)]
            prog.append((reads, mfmas))
    return prog


def qk_program(kslot, buf):
    """S^T[buf] = K Q^T: fragment (t, kt) = key half kt x d chunk pair t, shared by both row blocks"""
    prog = []
    for t in range(8):
        for kt in range(2):
            reads = [f'ds_read_b128 a[{{r0}}:{{r3}}], v{KA + t} offset:{kslot * TILE_BYTES + kt * 8192}']
            mfmas = [f'MFMA {s_acc(buf, rb, kt)}, a[{{r0}}:{{r3}}], {q_frag(rb, t)}, ' +
                     ('0' if t == 0 else s_acc(buf, rb, kt)) for rb in range(2)]
            prog.append((reads, mfmas))
    return prog


def mfma_block(prog, valu=(), valu_late=(), n_early=0, after=None):
    """The MFMAs of `prog` with their LDS reads LOOKAHEAD fragments ahead and exact waits.
    valu: vector instructions spread evenly between the MFMAs; valu_late: more of them that
    may only start once the first n_early fragments' MFMAs have been issued (they overwrite
    registers those MFMAs read); after: {k: instructions placed behind the k-th MFMA}."""
    after = after or {}
    V = list(valu) + list(valu_late)
    first_late = len(valu)
    n_mfma = 2 * len(prog)
    per = (len(V) + n_mfma) // (n_mfma + 1)
    pos = [0]

    def take(n):
        out = V[pos[0]:pos[0] + n]
        pos[0] += n
        return out
    issued = []   # fragment of every LDS read issued so far, in order
    L = []

    def issue(f):
        r = AF + 4 * (f % NSLOT)
        for rd in prog[f][0]:
            L.append(rd.format(r0=r, r1=r + 1, r2=r + 2, r3=r + 3))
            issued.append(f)
    for f in range(min(LOOKAHEAD, len(prog))):
        issue(f)
    L += take(min(per, first_late))
    k = 0
    for f in range(len(prog)):
        if f % WAIT_EVERY == 0:   # one wait covers this fragment and the next WAIT_EVERY - 1
            last = max(i for i, x in enumerate(issued) if x <= min(f + WAIT_EVERY - 1, len(prog) - 1))
            L.append(f's_waitcnt lgkmcnt({min(15, len(issued) - 1 - last)})')
        r = AF + 4 * (f % NSLOT)
        for i, mf in enumerate(prog[f][1]):
            L.append(mf.format(r0=r, r3=r + 3))
            if i == 0 and f + LOOKAHEAD < len(prog):
                issue(f + LOOKAHEAD)
            k += 1
            n = per if f >= n_early else min(per, max(0, first_late - pos[0]))
            L += take(n)
            L += after.get(k, [])
    L += take(len(V))
    return L + MFMA_DRAIN


def rescale(rb):
    """O^T of row block rb *= factor where the softmax raised the reference (skipped when no lane did)"""
    keep = label('keep')
    L = [f's_cmp_eq_u64 {S_RAISED[rb]}, 0', f's_cbranch_scc1 {keep}']
    for r0 in range(0, 64, 8):
        regs = [(AO + 64 * rb + r0 + i, TMP + i) for i in range(8)]
        L += [f'v_accvgpr_read_b32 v{t}, a{a}' for a, t in regs]
        L += [f'v_mul_f32 v{t}, v{t}, {V_C[rb]}' for a, t in regs]
        L += [f'v_accvgpr_write_b32 a{a}, v{t}' for a, t in regs]
    return L + [f'{keep}:']


def key_of_score(j):
    """key (inside the step, without the lane's 4*hg) of score register j of a row block"""
    return 32 * (j >> 4) + 8 * ((j & 15) >> 2) + (j & 3)


def mask_scores(buf):
    """scores of keys outside [rlo, rhi] of the lane's rows become -inf"""
    L = [f's_lshl_b32 s96, {S_B}, 6', f's_add_u32 s96, s96, {S_KEY_BEGIN}']
    for rb in range(2):
        no_win = label('nowin')
        L += [f'v_subrev_u32 v{V_RHI_REL}, s96, v{V_RHI[rb]}']
        for j in range(32):
            L += [f'v_cmp_gt_i32 vcc, {key_of_score(j)}, v{V_RHI_REL}',
                  f'v_cndmask_b32 {S(buf, rb, j)}, {S(buf, rb, j)}, {V_NINF}, vcc']
        L += [f's_cmp_eq_u32 {S_WINDOW}, 0', f's_cbranch_scc1 {no_win}', f'v_subrev_u32 v{V_RLO_REL}, s96, v{V_RLO[rb]}']
        for j in range(32):
            L += [f'v_cmp_lt_i32 vcc, {key_of_score(j)}, v{V_RLO_REL}',
                  f'v_cndmask_b32 {S(buf, rb, j)}, {S(buf, rb, j)}, {V_NINF}, vcc']
        L += [f'{no_win}:']
    return L


# ---------------------------------------------------------------------------------------
# copies of K and V tiles (global -> LDS, 16 bytes per lane) and their addresses
def copy1(offs, lds_imm, i, base):
    # M0 = LDS address of lane 0's 16 bytes; one idle state between writing M0 and the copy
    return [f's_add_u32 m0, {S_LDS_ROW0}, {lds_imm + i * 1024}', 's_nop 0',
            f'global_load_lds_dwordx4 v{offs[i]}, {base}']


def copy4(offs, lds_imm, base):
    return [l for i in range(4) for l in copy1(offs, lds_imm, i, base)]


def copy4_clamped(offs, lds_imm, base):
    """rows past s83 (last written row of the step) are fetched from row s83 instead"""
    a, b = V_TMP_COPY
    L = []
    for i in range(4):
        L += [f'v_lshrrev_b32 v{a}, 8, v{offs[i]}', f'v_min_u32 v{a}, s83, v{a}', f'v_lshlrev_b32 v{a}, 8, v{a}',
              f'v_and_b32 v{b}, 0xff, v{offs[i]}', f'v_or_b32 v{a}, v{a}, v{b}',
              f's_add_u32 m0, {S_LDS_ROW0}, {lds_imm + i * 1024}', 's_nop 0',
              f'global_load_lds_dwordx4 v{a}, {base}']
    return L


def copy_tile(offs, lds_imm, base, step_reg):
    """whole copy, or clamped if step_reg is past the last step with all 64 rows written"""
    clamp, done = label('clamp'), label('copied')
    L = [f's_cmp_gt_i32 {step_reg}, {S_WHOLE_HI}', f's_cbranch_scc1 {clamp}']
    L += copy4(offs, lds_imm, base) + [f's_branch {done}', f'{clamp}:']
    # s83 = last written row counted from the wave's first row of the (clamped) quarter, >= 0
    L += [f's_lshl2_add_u32 s83, {step_reg}, {S_STEP0}', f's_lshr_b32 s82, {S_LAST_ROW}, 4', 's_min_u32 s83, s83, s82',
          's_lshl_b32 s83, s83, 4', f's_sub_u32 s83, {S_LAST_ROW}, s83']
    return L + copy4_clamped(offs, lds_imm, base) + [f'{done}:']


def offset_of_step_b_plus_2():
    """s82 = the wave's quarter (16 keys, counted from the start of the sequence) of step b,
    S_PHYS = physical block of its quarter of step b+2 -> s[84:85] = byte offset of the wave's rows
    of that step (block * bytes per block + position inside the block; head excluded).  A quarter
    past the last written token is replaced by the one that holds it."""
    return ['s_add_u32 s83, s82, 8', f's_lshr_b32 s92, {S_LAST_ROW}, 4', 's_min_u32 s83, s83, s92',
            f's_and_b32 s83, s83, {S_SPB_MASK}', 's_lshl_b32 s83, s83, 12',
            f's_mul_hi_u32 s85, {S_PHYS}, {S_BLK_BYTES}', f's_mul_i32 s84, {S_PHYS}, {S_BLK_BYTES}',
            's_add_u32 s84, s84, s83', 's_addc_u32 s85, s85, 0']


def prefetch_block_id():
    """physical block of the wave's quarter of step min(b+3, n_steps-1), read through the scalar cache"""
    return [f's_add_u32 s83, {S_B}, 3', f's_sub_u32 s96, {S_NSTEPS}, 1', 's_min_u32 s83, s83, s96',
            f's_lshl2_add_u32 s83, s83, {S_STEP0}', f's_lshr_b32 s92, {S_LAST_ROW}, 4', 's_min_u32 s83, s83, s92',
            f's_lshr_b32 s83, s83, {S_SPB_SHIFT}', 's_lshl_b32 s83, s83, 2',
            f's_add_u32 s92, s{S_BT}, s83', f's_addc_u32 s93, s{S_BT + 1}, 0',
            f's_load_dword {S_PHYS}, s[92:93], 0x0']


def k_base():
    return [f's_add_u32 s86, s{S_KHEAD}, s84', f's_addc_u32 s87, s{S_KHEAD + 1}, s85']


def v_base():
    return [f's_add_u32 s52, s{S_VHEAD}, s90', f's_addc_u32 s53, s{S_VHEAD + 1}, s91']


def rotate_offsets():
    return [f's_mov_b64 {S_OFF0}, {S_OFF1}', f's_mov_b64 {S_OFF1}, s[84:85]']


def hand_over_begin():
    # own copies landed and own LDS reads done, then everybody's
    return ['s_waitcnt vmcnt(0) lgkmcnt(0)', 's_barrier', f's_lshl2_add_u32 s82, {S_B}, {S_STEP0}']


def hand_over_steady():
    """addresses only (K tile at s[86:87], V tile at s[52:53]); the copies themselves are spread
    through the MFMAs that follow, so that the four waves of a workgroup do not queue 32 KB of
    copies at the same moment behind the barrier"""
    return (hand_over_begin() + offset_of_step_b_plus_2() + k_base() + v_base() + rotate_offsets() +
            prefetch_block_id())


def steady_copies(sub):
    """K(b+2) behind MFMAs 2, 4, 6, 8 and V(b) behind MFMAs 10, 12, 14, 16"""
    after = {2 + 2 * i: copy1(KOFF, sub * TILE_BYTES, i, 's[86:87]') for i in range(4)}
    after.update({10 + 2 * i: copy1(VOFF, V_RING + sub * TILE_BYTES, i, S_VBASE) for i in range(4)})
    return after


def hand_over_general(sub):
    """iteration b, b & 1 = sub: K(b+2) -> K slot sub, V(b) -> V slot sub (both last read in iteration b-1)"""
    no_k, no_v = label('nok'), label('nov')
    L = hand_over_begin()
    L += [f's_add_u32 s96, {S_B}, 2', f's_cmp_ge_i32 s96, {S_NSTEPS}', f's_cbranch_scc1 {no_k}']
    L += offset_of_step_b_plus_2() + k_base() + copy_tile(KOFF, sub * TILE_BYTES, 's[86:87]', 's96') + [f'{no_k}:']
    L += [f's_cmp_ge_i32 {S_B}, {S_NSTEPS}', f's_cbranch_scc1 {no_v}']
    L += v_base() + copy_tile(VOFF, V_RING + sub * TILE_BYTES, S_VBASE, S_B) + [f'{no_v}:']
    return L + rotate_offsets() + prefetch_block_id()


# ---------------------------------------------------------------------------------------
def unless_active(reg, skip):
    """branch to skip unless first active step <= reg <= last active step of the wave"""
    return [f's_cmp_lt_i32 {reg}, {S_JFIRST}', f's_cbranch_scc1 {skip}',
            f's_cmp_gt_i32 {reg}, {S_JLAST}', f's_cbranch_scc1 {skip}']


def general_iteration(sub):
    """iteration b (b & 1 = sub): PV(b-1), softmax(b) -> P, QK(b+1), each only if its step is active"""
    no_pv, no_s, no_qk, do_mask, no_mask = (label(n) for n in ('nopv', 'nos', 'noqk', 'mask', 'nomask'))
    L = hand_over_general(sub)
    L += [f's_sub_u32 s96, {S_B}, 1'] + unless_active('s96', no_pv) + mfma_block(pv_program(1 - sub)) + [f'{no_pv}:']
    L += unless_active(S_B, no_s)
    L += [f's_cmp_lt_i32 {S_B}, {S_NOMASK_LO}', f's_cbranch_scc1 {do_mask}',
          f's_cmp_gt_i32 {S_B}, {S_NOMASK_HI}', f's_cbranch_scc1 {do_mask}', f's_branch {no_mask}']
    L += [f'{do_mask}:'] + mask_scores(sub) + [f'{no_mask}:']
    probs, pack = softmax(sub)
    L += probs + pack + rescale(0) + rescale(1) + [f'{no_s}:']
    L += [f's_add_u32 s96, {S_B}, 1'] + unless_active('s96', no_qk) + mfma_block(qk_program(1 - sub, 1 - sub)) + [f'{no_qk}:']
    return L + [f's_add_u32 {S_B}, {S_B}, 1']


def steady_iteration(sub):
    """all three parts active, step b unmasked, every copy whole: the 64 MFMAs of PV(b-1) and
    QK(b+1) in one stream with the vector work of softmax(b) between them"""
    probs, pack = softmax(sub)
    prog = pv_program(1 - sub) + qk_program(1 - sub, 1 - sub)
    L = hand_over_steady() + mfma_block(prog, probs, pack, n_early=16, after=steady_copies(sub))
    return L + rescale(0) + rescale(1) + [f's_add_u32 {S_B}, {S_B}, 1']


def prologue():
    """Q^T into accumulation registers, O^T = 0, K(0) and K(1) on their way, QK(0)"""
    no_k1, no_qk = label('nok1'), label('noqk0')
    L = []
    for rb in range(2):
        for t in range(8):
            r = SB[0] + 32 * rb + 4 * t
            L.append(f'global_load_dwordx4 v[{r}:{r + 3}], v[{V_Q[rb]}:{V_Q[rb] + 1}], off offset:{32 * t}')
    L += [f'v_accvgpr_write_b32 a{AO + r}, 0' for r in range(128)]
    L += [f'v_mov_b32 {V_M[rb]}, 0xf149f2ca' for rb in range(2)]      # -1e30
    L += [f'v_mov_b32 {V_L[rb]}, 0' for rb in range(2)] + [f'v_mov_b32 {V_C[rb]}, 0' for rb in range(2)]
    L += [f'v_mov_b32 {V_NINF}, 0xff800000', 's_waitcnt vmcnt(0)']
    L += [f'v_accvgpr_write_b32 a{AQ + i}, v{SB[0] + i}' for i in range(64)]
    # K(0) -> K slot 0, K(1) -> K slot 1
    L += ['s_mov_b32 s96, 0', f's_add_u32 s86, s{S_KHEAD}, s90', f's_addc_u32 s87, s{S_KHEAD + 1}, s91']
    L += copy_tile(KOFF, 0, 's[86:87]', 's96')
    L += ['s_mov_b32 s96, 1', f's_cmp_ge_i32 s96, {S_NSTEPS}', f's_cbranch_scc1 {no_k1}']
    L += [f's_add_u32 s86, s{S_KHEAD}, s98', f's_addc_u32 s87, s{S_KHEAD + 1}, s99']
    L += copy_tile(KOFF, TILE_BYTES, 's[86:87]', 's96') + [f'{no_k1}:']
    L += ['s_waitcnt vmcnt(0) lgkmcnt(0)', 's_barrier', 's_mov_b32 s96, 0']
    L += unless_active('s96', no_qk) + mfma_block(qk_program(0, 0)) + [f'{no_qk}:']
    return L


def epilogue():
    """Normal mode: O^T / l, rounded, to the lane's output rows.  Partial mode (the tile's key
    range was split across workgroups): O^T as it is, the reference m and the sum l, in fp32, to
    the lane's rows of the partial-result buffer (a row there is O^T, 128 floats, then m and l at
    byte 512; the caller spaces the rows).  Accumulator mt, register r of a row block is
    column 32 mt + 8 (r / 4) + 4 hg + r % 4; the row addresses already include the lane's 4 hg
    columns."""
    partial, end = label('partial'), label('end')
    L = [f's_cmp_eq_u32 {S_PARTIAL}, 0', f's_cbranch_scc0 {partial}']
    for mode in ('normal', 'partial'):
        if mode == 'partial':
            L += [f's_branch {end}', f'{partial}:']
        for rb in range(2):
            t, inv = TMP + 8, TMP + 9
            # the other half-wave holds the sum over the other 32 keys of every step
            L += [f'v_mov_b32 v{t}, {V_L[rb]}', 's_nop 1', f'v_permlane32_swap_b32 v{t}, {V_L[rb]}',
                  f'v_add_f32 v{t}, v{t}, {V_L[rb]}']
            if mode == 'normal':
                L += [f'v_rcp_f32 v{inv}, v{t}', f's_mov_b64 exec, {S_LIVE[rb]}']
            else:
                L += [f'v_mov_b32 v{TMP + 10}, {V_M[rb]}', f'v_mov_b32 v{TMP + 11}, v{t}', f's_mov_b64 exec, {S_LIVE[rb]}',
                      f'global_store_dwordx2 v[{V_OUT[rb]}:{V_OUT[rb] + 1}], v[{TMP + 10}:{TMP + 11}], off offset:512']
            for mt in range(4):
                for rq in range(4):
                    a0 = AO + 64 * rb + 16 * mt + 4 * rq
                    d = [TMP + 4 * (rq & 1) + i for i in range(4)]
                    L += [f'v_accvgpr_read_b32 v{d[i]}, a{a0 + i}' for i in range(4)]
                    if mode == 'normal':
                        L += [f'v_mul_f32 v{d[i]}, v{d[i]}, v{inv}' for i in range(4)]
                        L += [f'CVT v{d[0]}, v{d[0]}, v{d[1]}', f'CVT v{d[1]}, v{d[2]}, v{d[3]}',
                              f'global_store_dwordx2 v[{V_OUT[rb]}:{V_OUT[rb] + 1}], v[{d[0]}:{d[1]}], off offset:{64 * mt + 16 * rq}']
                    else:
                        L += ['s_nop 0',
                              f'global_store_dwordx4 v[{V_OUT[rb]}:{V_OUT[rb] + 1}], v[{d[0]}:{d[3]}], off offset:{128 * mt + 32 * rq}']
            L += ['s_mov_b64 exec, -1']
    return L + [f'{end}:']


def tile():
    even, even_body, odd, steady, done = (f'.Lfsf_{n}_%=' for n in ('g0', 'g0body', 'g1', 'fast', 'done'))
    L = prologue()
    L += [f'{even}:', f's_cmp_gt_i32 {S_B}, {S_NSTEPS}', f's_cbranch_scc1 {done}']
    # an even b with fast_lo <= b and b + 1 <= fast_hi: run steady pairs up to fast_hi
    L += [f's_cmp_lt_i32 {S_B}, {S_FAST_LO}', f's_cbranch_scc1 {even_body}',
          f's_add_u32 s96, {S_B}, 1', f's_cmp_gt_i32 s96, {S_FAST_HI}', f's_cbranch_scc1 {even_body}',
          f's_sub_u32 {S_PAIRS}, {S_FAST_HI}, {S_B}', f's_add_u32 {S_PAIRS}, {S_PAIRS}, 1',
          f's_lshr_b32 {S_PAIRS}, {S_PAIRS}, 1', f'{steady}:']
    L += steady_iteration(0) + steady_iteration(1)
    L += [f's_sub_u32 {S_PAIRS}, {S_PAIRS}, 1', f's_cmp_lg_u32 {S_PAIRS}, 0', f's_cbranch_scc1 {steady}',
          f's_branch {even}']
    L += [f'{even_body}:'] + general_iteration(0)
    L += [f'{odd}:', f's_cmp_gt_i32 {S_B}, {S_NSTEPS}', f's_cbranch_scc1 {done}'] + general_iteration(1)
    L += [f's_branch {even}', f'{done}:']
    return L + epilogue()


HEADER = """\
// Generated by gen_prefill_sequence.py -- do not edit; change the generator and run it again.
// The instruction sequence of one prompt-chunk tile (see attn_prefill_body.h).
#pragma once

"""


def clobbers():
    """registers the sequence writes that are not operands of the asm statement"""
    v = list(V_TMP_COPY) + [V_RHI_REL, V_RLO_REL] + list(range(44, 50)) + [51]
    v += list(range(SB[0], PB + 32)) + list(range(TMP, 256))
    s = [52, 53, 54, 55] + list(range(82, 90)) + [92, 93, 95, 96]
    names = [f'"s{r}"' for r in s] + [f'"v{r}"' for r in v] + [f'"a{r}"' for r in range(256)]
    rows = [', '.join(names[i:i + 12]) for i in range(0, len(names), 12)]
    return '#define FSF_TILE_CLOBBERS \\\n  ' + ', \\\n  '.join(rows) + '\n'


def render():
    _uid[0] = 0
    lines = tile()
    out = [HEADER + clobbers() + '\n#define FSF_TILE_SEQUENCE(MFMA, CVT) \\']
    for k, l in enumerate(lines):
        cont = ' \\' if k + 1 < len(lines) else ''
        if l.endswith(':'):
            out.append(f'  "{l}\\n"{cont}')
        elif l.startswith('MFMA '):
            out.append(f'  MFMA "{l[4:]}\\n\\t"{cont}')
        elif l.startswith('CVT '):
            out.append(f'  CVT "{l[3:]}\\n\\t"{cont}')
        else:
            out.append(f'  "{l}\\n\\t"{cont}')
    return '\n'.join(out) + '\n'


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), 'attn_prefill_sequence.h')
    text = render()
    if '--check' in sys.argv[1:]:
        with open(path) as f:
            ok = f.read() == text
        print('up to date' if ok else f'{path} does not match the generator')
        sys.exit(0 if ok else 1)
    with open(path, 'w') as f:
        f.write(text)
    print(f'wrote {path}: {text.count(chr(10))} lines')


if __name__ == '__main__':
    main()
