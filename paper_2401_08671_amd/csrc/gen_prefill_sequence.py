#!/usr/bin/env python3
"""Writes attn_prefill_sequence.h: the fixed gfx950 instruction sequence a wave runs to walk
one prompt-chunk tile over its 64-key steps (macro FSF_TILE_SEQUENCE, used by
attn_prefill_body.h, which documents the algorithm, the LDS layout and the register map).

    python gen_prefill_sequence.py            # rewrites the header next to this file
    python gen_prefill_sequence.py --check    # exit 1 if the header on disk is out of date

The sequence is emitted as the string of one inline-asm statement.  Two tokens stay macro
parameters so that one sequence serves both element types: MFMA (the 32x32x16 matrix
instruction) and CVT (the packing float -> 2-byte conversion).
"""
import os
import sys

# ---- register map (vector)
V_TMP_COPY = (28, 29)       # temporaries of a clamped copy
V_RHI, V_RLO = 32, 33       # last / first visible key of the lane's row, minus 4*hg
V_RHI_REL, V_RLO_REL = 34, 35   # the same relative to the first key of the step
VOFF = [36, 37, 38, 39]     # lane offsets of the wave's four V copy instructions
V_M, V_L, V_C, V_SL2 = 'v40', 'v41', 'v42', 'v43'   # running max, running sum, rescale factor, scale*log2(e)
KOFF = [44, 45, 46, 47]     # ... of its four K copy instructions
V_NINF = 'v48'
VA = 50                     # v50..v53: LDS address of the lane's V^T fragment, per 32-wide d tile
KA = 54                     # v54..v61: LDS address of the lane's K fragment, per k-step
QF = 62                     # v62..v93: Q^T fragments
ACC = 94                    # v94..v157: O^T, four 32x32 accumulators
SC = 158                    # v158..v189: S^T, two 32x32 accumulators
PF = [190, 206]             # the two P^T buffers, 16 registers each
TMP = 222                   # v222..v231: softmax temporaries
T0, NFRAG = 232, 6          # v232..v255: six 4-register K / V^T fragments in flight
# ---- register map (scalar)
S_NSTEPS, S_JFIRST, S_JLAST = 's60', 's61', 's62'
S_NOMASK_LO, S_NOMASK_HI = 's63', 's64'
S_FAST_LO, S_FAST_HI, S_WHOLE_HI = 's65', 's66', 's67'
S_LAST_ROW, S_KEY_BEGIN, S_WINDOW, S_STEP0 = 's68', 's69', 's70', 's71'
S_SPB_MASK, S_SPB_SHIFT = 's72', 's73'
S_BT, S_KHEAD, S_VHEAD = 74, 76, 78      # 64-bit pairs
S_BLK_BYTES, S_LDS_ROW0 = 's80', 's81'
S_RAISED = 's[88:89]'       # lanes whose reference was raised by the softmax of this step
S_PHYS_NEXT, S_PAIRS, S_B = 's94', 's95', 's97'
# s82..s87, s92, s93, s96, s98, s99: temporaries;  s[90:91]: byte offset of step b's tiles

TILE_BYTES = 16384          # one K or V tile in LDS
V_RING = 2 * TILE_BYTES     # K slots at 0 and 16384, V slots at 32768 and 49152
MFMA_DRAIN = ['s_nop 7', 's_nop 3']   # idle cycles before vector code may read the last MFMA's result

_uid = [0]


def label(name):
    _uid[0] += 1
    return f'.Lfsf_{name}{_uid[0]}_%='


def acc(mt):
    return f'v[{ACC + 16 * mt}:{ACC + 16 * mt + 15}]'


def sc(kt):
    return f'v[{SC + 16 * kt}:{SC + 16 * kt + 15}]'


def qf(t):
    return f'v[{QF + 4 * t}:{QF + 4 * t + 3}]'


def pf(buf, u):
    return f'v[{PF[buf] + 4 * u}:{PF[buf] + 4 * u + 3}]'


# ---------------------------------------------------------------------------------------
# S^T = K Q^T of one step: 8 k-steps x 2 key halves, K fragments read three k-steps ahead
def qk(kslot, after=None):
    """`after`: {k-step t: instructions to place behind its two MFMAs} (no vector ALU work on
    the scores or fragments; scalar and copy instructions are fine)"""
    after = after or {}
    kb = kslot * TILE_BYTES
    ahead = NFRAG // 2
    frag = lambda t, kt: T0 + ((t % ahead) * 2 + kt) * 4
    read = lambda t, kt: f'ds_read_b128 v[{frag(t, kt)}:{frag(t, kt) + 3}], v{KA + t} offset:{kb + kt * 8192}'
    L = [read(t, kt) for t in range(ahead) for kt in range(2)]
    for t in range(8):
        L.append(f's_waitcnt lgkmcnt({2 * min(ahead - 1, 7 - t)})')
        for kt in range(2):
            c = '0' if t == 0 else sc(kt)
            L.append(f'MFMA {sc(kt)}, v[{frag(t, kt)}:{frag(t, kt) + 3}], {qf(t)}, {c}')
        if t + ahead < 8:
            L += [read(t + ahead, kt) for kt in range(2)]
        L += after.get(t, [])
    return L + MFMA_DRAIN


# O^T += V^T P^T of one step: MFMA i covers k-step u = i / 4 (16 keys), d tile mt = i % 4
def pv_reads(i, vslot):
    vb = vslot * TILE_BYTES   # va[] already points into the V ring
    u, mt = i >> 2, i & 3
    r = T0 + (i % NFRAG) * 4
    return [f'ds_read_b64_tr_b16 v[{r}:{r + 1}], v{VA + mt} offset:{vb + 16 * u * 256}',
            f'ds_read_b64_tr_b16 v[{r + 2}:{r + 3}], v{VA + mt} offset:{vb + (16 * u + 8) * 256}']


def pv_mfma(i, buf):
    u, mt = i >> 2, i & 3
    r = T0 + (i % NFRAG) * 4
    return [f's_waitcnt lgkmcnt({2 * min(NFRAG - 1, 15 - i)})',
            f'MFMA {acc(mt)}, v[{r}:{r + 3}], {pf(buf, u)}, {acc(mt)}']


def pv(buf, vslot, between=None):
    """P^T from buffer buf, V from slot vslot; `between` = vector instructions to spread
    between the MFMAs (they must not touch the accumulators, buffer buf or the fragments)."""
    V = list(between or [])
    per = (len(V) + 16) // 17
    pos = [0]

    def take(n):
        out = V[pos[0]:pos[0] + n]
        pos[0] += n
        return out
    L = []
    for i in range(NFRAG):
        L += pv_reads(i, vslot)
    L += take(per)
    for i in range(16):
        L += pv_mfma(i, buf)
        if i + NFRAG < 16:
            L += pv_reads(i + NFRAG, vslot)
        L += take(per if i < 15 else len(V))
    return L + MFMA_DRAIN


def softmax(new):
    """Online softmax of the step's scores (already masked where needed) -> P^T buffer `new`.
    A lane holds 32 scores of one row; the other half-wave holds the row's other 32."""
    e = [TMP + i for i in range(8)]
    t = e[4:]
    sa, sb = TMP + 8, TMP + 9
    S = lambda j: f'v{SC + j}'
    V = [f'v_max3_f32 v{t[c]}, {S(3 * c)}, {S(3 * c + 1)}, {S(3 * c + 2)}' for c in range(4)]
    j, c = 12, 0
    while j + 1 < 32:
        V.append(f'v_max3_f32 v{t[c]}, v{t[c]}, {S(j)}, {S(j + 1)}')
        j += 2
        c = (c + 1) % 4
    V += [f'v_max3_f32 v{t[0]}, v{t[0]}, v{t[1]}, v{t[2]}',
          f'v_max_f32 v{t[0]}, v{t[0]}, v{t[3]}',
          f'v_mov_b32 v{t[1]}, v{t[0]}',
          's_nop 1',
          f'v_permlane32_swap_b32 v{t[1]}, v{t[0]}',
          f'v_max_f32 v{t[0]}, v{t[0]}, v{t[1]}',
          # raise the running reference only where the maximum outgrew it by more than 2^8
          f'v_mul_f32 v{t[0]}, {V_SL2}, v{t[0]}',
          f'v_max_f32 v{t[1]}, v{t[0]}, {V_M}',
          f'v_sub_f32 v{t[2]}, v{t[1]}, {V_M}',
          f'v_cmp_lt_f32 vcc, 0x41000000, v{t[2]}',
          f'v_cndmask_b32 v{t[1]}, {V_M}, v{t[1]}, vcc',
          f's_mov_b64 {S_RAISED}, vcc',
          f'v_sub_f32 v{t[2]}, {V_M}, v{t[1]}',
          f'v_exp_f32 {V_C}, v{t[2]}',
          f'v_mov_b32 {V_M}, v{t[1]}',
          f'v_mov_b32 v{sa}, 0',
          f'v_mov_b32 v{sb}, 0',
          f'v_mul_f32 {V_L}, {V_L}, {V_C}']
    # probabilities, their sum, and the packed operand: P^T register r = pack(p[2r], p[2r+1])
    for g in range(8):
        ee = e[:4] if g % 2 == 0 else e[4:]
        js = [4 * g + i for i in range(4)]
        V += [f'v_fma_f32 v{ee[i]}, {S(js[i])}, {V_SL2}, -{V_M}' for i in range(4)]
        V += [f'v_exp_f32 v{ee[i]}, v{ee[i]}' for i in range(4)]
        V += [f'v_add_f32 v{sa}, v{sa}, v{ee[0]}',
              f'v_add_f32 v{sb}, v{sb}, v{ee[1]}',
              f'CVT v{PF[new] + 2 * g}, v{ee[0]}, v{ee[1]}',
              f'v_add_f32 v{sa}, v{sa}, v{ee[2]}',
              f'v_add_f32 v{sb}, v{sb}, v{ee[3]}',
              f'CVT v{PF[new] + 2 * g + 1}, v{ee[2]}, v{ee[3]}']
    V += [f'v_add_f32 v{sa}, v{sa}, v{sb}', f'v_add_f32 {V_L}, {V_L}, v{sa}']
    return V


def rescale():
    """O^T *= factor where the softmax raised the reference (skipped when no lane did)."""
    keep = label('keep')
    return ([f's_cmp_eq_u64 {S_RAISED}, 0', f's_cbranch_scc1 {keep}'] +
            [f'v_mul_f32 v{ACC + r}, v{ACC + r}, {V_C}' for r in range(64)] + [f'{keep}:'])


def key_of_score(j):
    """key (inside the step, without the lane's 4*hg) of score register j"""
    return 32 * (j >> 4) + 8 * ((j & 15) >> 2) + (j & 3)


def mask_scores():
    """scores of keys outside [rlo, rhi] of the lane's row become -inf"""
    no_win = label('nowin')
    L = [f's_lshl_b32 s96, {S_B}, 6', f's_add_u32 s96, s96, {S_KEY_BEGIN}', f'v_subrev_u32 v{V_RHI_REL}, s96, v{V_RHI}']
    for j in range(32):
        L += [f'v_cmp_gt_i32 vcc, {key_of_score(j)}, v{V_RHI_REL}', f'v_cndmask_b32 v{SC + j}, v{SC + j}, {V_NINF}, vcc']
    L += [f's_cmp_eq_u32 {S_WINDOW}, 0', f's_cbranch_scc1 {no_win}', f'v_subrev_u32 v{V_RLO_REL}, s96, v{V_RLO}']
    for j in range(32):
        L += [f'v_cmp_lt_i32 vcc, {key_of_score(j)}, v{V_RLO_REL}', f'v_cndmask_b32 v{SC + j}, v{SC + j}, {V_NINF}, vcc']
    return L + [f'{no_win}:']


# ---------------------------------------------------------------------------------------
# hand-over: copies of the next tiles, address arithmetic on the scalar unit
def copy1(offs, lds_imm, i, base='s[86:87]'):
    # M0 = LDS address of lane 0's 16 bytes; one idle state between writing M0 and the copy
    return [f's_add_u32 m0, {S_LDS_ROW0}, {lds_imm + i * 1024}', 's_nop 0',
            f'global_load_lds_dwordx4 v{offs[i]}, {base}']


def copy4(offs, lds_imm):
    return [l for i in range(4) for l in copy1(offs, lds_imm, i)]


def copy4_clamped(offs, lds_imm):
    """rows past s83 (last written row of the step) are fetched from row s83 instead"""
    a, b = V_TMP_COPY
    L = []
    for i in range(4):
        L += [f'v_lshrrev_b32 v{a}, 8, v{offs[i]}', f'v_min_u32 v{a}, s83, v{a}', f'v_lshlrev_b32 v{a}, 8, v{a}',
              f'v_and_b32 v{b}, 0xff, v{offs[i]}', f'v_or_b32 v{a}, v{a}, v{b}',
              f's_add_u32 m0, {S_LDS_ROW0}, {lds_imm + i * 1024}', 's_nop 0',
              f'global_load_lds_dwordx4 v{a}, s[86:87]']
    return L


def offset_of_next_step():
    """s82 = step b's index in the sequence -> s[84:85] = byte offset of step b+1's tiles
    (physical block * bytes per block + position inside the block; head excluded)"""
    return ['s_add_u32 s83, s82, 1', f's_and_b32 s83, s83, {S_SPB_MASK}', 's_lshl_b32 s83, s83, 14',
            f's_mul_hi_u32 s85, {S_PHYS_NEXT}, {S_BLK_BYTES}', f's_mul_i32 s84, {S_PHYS_NEXT}, {S_BLK_BYTES}',
            's_add_u32 s84, s84, s83', 's_addc_u32 s85, s85, 0']


def prefetch_block_id():
    """physical block of step b+2 (s82 = step b's index in the sequence)"""
    return ['s_add_u32 s83, s82, 2', f's_lshr_b32 s83, s83, {S_SPB_SHIFT}', 's_lshl_b32 s83, s83, 2',
            f's_add_u32 s92, s{S_BT}, s83', f's_addc_u32 s93, s{S_BT + 1}, 0',
            f's_load_dword {S_PHYS_NEXT}, s[92:93], 0x0']


def k_base():
    return [f's_add_u32 s86, s{S_KHEAD}, s84', f's_addc_u32 s87, s{S_KHEAD + 1}, s85']


def v_base(lo='s86', hi='s87'):
    return [f's_add_u32 {lo}, s{S_VHEAD}, s90', f's_addc_u32 {hi}, s{S_VHEAD + 1}, s91']


def hand_over_begin():
    # own copies landed and own LDS reads done, then everybody's
    return ['s_waitcnt vmcnt(0) lgkmcnt(0)', 's_barrier', f's_add_u32 s82, {S_STEP0}, {S_B}']


def hand_over_steady():
    """addresses only (K base in s[86:87], V base in s[98:99]); the copies themselves are spread
    through the first product, so that the four waves of a workgroup do not queue 32 KB of
    copies at the same moment behind the barrier"""
    L = hand_over_begin() + offset_of_next_step() + k_base() + v_base('s98', 's99')
    return L + ['s_mov_b64 s[90:91], s[84:85]'] + prefetch_block_id()


def steady_copies(sub):
    """K(b+1) behind k-steps 0..3 of QK(b), V(b) behind k-steps 4..7"""
    kslot, vslot = (sub + 1) & 1, sub & 1
    after = {i: copy1(KOFF, kslot * TILE_BYTES, i) for i in range(4)}
    after.update({4 + i: copy1(VOFF, V_RING + vslot * TILE_BYTES, i, 's[98:99]') for i in range(4)})
    return after


def hand_over_general(sub):
    kslot, vslot = (sub + 1) & 1, sub & 1
    no_k, k_clamp, k_done = label('nok'), label('kclamp'), label('kdone')
    no_v, v_clamp, v_done = label('nov'), label('vclamp'), label('vdone')
    no_p = label('nop')
    L = hand_over_begin()
    # K(b+1), if there is such a step; clamped if the step holds unwritten rows
    L += [f's_add_u32 s96, {S_B}, 1', f's_cmp_ge_i32 s96, {S_NSTEPS}', f's_cbranch_scc1 {no_k}']
    L += offset_of_next_step() + k_base() + [f's_cmp_gt_i32 s96, {S_WHOLE_HI}', f's_cbranch_scc1 {k_clamp}']
    L += copy4(KOFF, kslot * TILE_BYTES) + [f's_branch {k_done}', f'{k_clamp}:']
    L += ['s_lshl_b32 s83, s96, 6', f's_sub_i32 s83, {S_LAST_ROW}, s83']
    L += copy4_clamped(KOFF, kslot * TILE_BYTES) + [f'{k_done}:', f'{no_k}:']
    # V(b)
    L += [f's_cmp_ge_i32 {S_B}, {S_NSTEPS}', f's_cbranch_scc1 {no_v}']
    L += v_base() + [f's_cmp_gt_i32 {S_B}, {S_WHOLE_HI}', f's_cbranch_scc1 {v_clamp}']
    L += copy4(VOFF, V_RING + vslot * TILE_BYTES) + [f's_branch {v_done}', f'{v_clamp}:']
    L += [f's_lshl_b32 s83, {S_B}, 6', f's_sub_i32 s83, {S_LAST_ROW}, s83']
    L += copy4_clamped(VOFF, V_RING + vslot * TILE_BYTES) + [f'{v_done}:', f'{no_v}:']
    L += ['s_mov_b64 s[90:91], s[84:85]']
    L += [f's_add_u32 s96, {S_B}, 2', f's_cmp_ge_i32 s96, {S_NSTEPS}', f's_cbranch_scc1 {no_p}']
    return L + prefetch_block_id() + [f'{no_p}:']


# ---------------------------------------------------------------------------------------
def unless_active(reg, skip):
    """branch to skip unless first active step <= reg <= last active step of the wave"""
    return [f's_cmp_lt_i32 {reg}, {S_JFIRST}', f's_cbranch_scc1 {skip}',
            f's_cmp_gt_i32 {reg}, {S_JLAST}', f's_cbranch_scc1 {skip}']


def general_iteration(sub):
    no_qk, no_pv, no_s, do_mask, no_mask = (label(n) for n in ('noqk', 'nopv', 'nos', 'mask', 'nomask'))
    L = hand_over_general(sub)
    L += unless_active(S_B, no_qk) + qk(sub) + [f'{no_qk}:']
    L += [f's_sub_u32 s96, {S_B}, 1'] + unless_active('s96', no_pv) + pv(sub, (sub + 1) & 1) + [f'{no_pv}:']
    L += unless_active(S_B, no_s)
    L += [f's_cmp_lt_i32 {S_B}, {S_NOMASK_LO}', f's_cbranch_scc1 {do_mask}',
          f's_cmp_gt_i32 {S_B}, {S_NOMASK_HI}', f's_cbranch_scc1 {do_mask}', f's_branch {no_mask}']
    L += [f'{do_mask}:'] + mask_scores() + [f'{no_mask}:']
    L += softmax(1 - sub) + rescale() + [f'{no_s}:']
    return L + [f's_add_u32 {S_B}, {S_B}, 1']


def steady_iteration(sub):
    L = hand_over_steady() + qk(sub, steady_copies(sub))
    L += pv(sub, (sub + 1) & 1, between=softmax(1 - sub)) + rescale()
    return L + [f's_add_u32 {S_B}, {S_B}, 1']


def tile():
    even, even_body, odd, steady, done = (f'.Lfsf_{n}_%=' for n in ('g0', 'g0body', 'g1', 'fast', 'done'))
    L = [f'{even}:', f's_cmp_gt_i32 {S_B}, {S_NSTEPS}', f's_cbranch_scc1 {done}']
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
    return L + [f's_branch {even}', f'{done}:']


HEADER = """\
// Generated by gen_prefill_sequence.py -- do not edit; change the generator and run it again.
// The instruction sequence of one prompt-chunk tile (see attn_prefill_body.h).
#pragma once

"""


def render():
    lines = tile()
    out = [HEADER + '#define FSF_TILE_SEQUENCE(MFMA, CVT) \\']
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
