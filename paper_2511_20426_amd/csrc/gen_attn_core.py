#!/usr/bin/env python3
"""Emits attn_core_gfx950.inc: the hand-scheduled main loop of the bf16 cascaded-attention kernel.

The loop is written as one inline-assembly block (included by attn_bf16.hip) because its speed
rests on two things a compiler will not hold still for:

  * issue order -- a wave issues in order and an MFMA occupies the matrix pipe for 32 cycles, so
    every MFMA must be followed by ~28 cycles of independent VALU / LDS issue (the softmax of the
    previous tile, the operand prefetch) instead of by another MFMA;
  * register files -- Q fragments and the O^T accumulators live in AGPRs, which VALU code never
    touches in the loop; S^T tiles, P^T and the K/V operand fragments live in VGPRs.

Pipeline (a "step" is 32 keys, a page is 4 steps; t counts steps):
    QK(t+1): 16 MFMAs  S_next = K_frag x Q                      (K fragments from LDS)
    SM(t)  : p = exp2(S_cur), bf16 pack, row sums                (VALU; S_cur already holds
             s*c - m_ref: Q is pre-scaled by c = log2(e)/sqrt(D) and QK starts from -m_ref)
    PV(t-1): 16 MFMAs  O^T   += V_frag x P_prev                  (V fragments from LDS)
The three are independent inside a step.  K and V pages stream global -> LDS (no registers) into
two 2-page rings; per page there is one barrier that publishes V(q) and frees V(q-1)'s slot
(step 1, slot 0) and one that publishes K(q+1) and frees K(q)'s slot (step 2, slot 24).

Register map (fixed):
  a[0:127]    O^T accumulators, tile (mt, nt) at a[16*(2*mt+nt) ..]
  a[128:191]  Q fragments, (nt, ks) at a[128 + 4*(8*nt+ks) ..]
  v[0:31]     S tile A (nt 0: v0.., nt 1: v16..)     v[32:63]  S tile B
  v[64:79]    P^T tile A, (nt, kk) at v[64 + 4*(2*nt+kk) ..]      v[80:95]  P^T tile B
  v[96:127]   ring of 8 operand fragments
  v[128:135]  LDS address of chunk pair j in the K ring, v[136:143] the same in the V ring
  v148..v151  row-sum accumulators (column tile, parity of the element)
  v[184:199], v[200:215]  -m_ref of column tile 0 / 1, replicated 16 times: the C operand of the
              first MFMA of every S tile, so a tile comes out of the matrix pipe as s*c - m_ref
  v152..v175  temporaries
  v[216:223]  lane's byte offset inside a page for page load i = 0..7
  v177,v178   per-KV-block page-0 offsets (lane i = block i), low / high word
  v179        4*(lane/32): first key row this lane holds in a 32x32 accumulator
  v180        4*(lane ^ 32): ds_bpermute address of the lane holding the other half of this row
"""
from __future__ import annotations

import os
import sys

# Timing experiments only (CA_ABL in the environment of the build): switch parts of the loop off.
# 1 no softmax arithmetic, 2 no LDS operand reads, 4 no page loads, 8 no barriers.  Results are
# then meaningless; the shipped library is always built with 0.
ABL = int(os.environ.get("CA_ABL", "0"))

D_AHEAD = 4          # operand fragments are read this many MFMA pairs ahead of use
PAGE = 32768
VRING = 65536

# ---------------------------------------------------------------------------- register names
def V(n, w=1):
    return f"v{n}" if w == 1 else f"v[{n}:{n + w - 1}]"


def A(n, w=1):
    return f"a{n}" if w == 1 else f"a[{n}:{n + w - 1}]"


S_TILE = {"A": 0, "B": 32}
P_TILE = {"A": 64, "B": 80}
FR = 96
XOK, XOV = 128, 136
LACC = 148
NT = [184, 200]      # -m_ref replicated 16x per column tile
TMP = 152            # 152..175
T_FMA = [152, 153]
PX = [154, 155, 156, 157]
MX = [158, 159]
RT = list(range(160, 176))     # rare-path temporaries
TBLLO, TBLHI, KIDX, XLANE = 177, 178, 179, 180
DMAOFF = 216         # 216..223: lane's byte offset in a page for load i (+4096 i)

# scalar registers (all inside the clobbered range s36..s95)
S_NLEFT, S_P, S_PM1, S_STRIDE, S_NKVB = 41, 42, 43, 44, 45
S_POOL = 46          # 46,47
S_M0B, S_LASTV = 48, 49
S_VLAST = 50         # 50..53
S_PGCUR, S_PGNEXT = 54, 55
S_KKB, S_KPG, S_VKB, S_VPG = 56, 57, 58, 59
S_T = 60             # 60..69 temporaries
S_ADDR = 70          # 70,71
S_VCC = 72           # 72,73
S_LDS0 = 74


class Emitter:
    def __init__(self):
        self.lines = []
        self.cold = []       # out-of-line blocks, appended after the loop
        self.uid = 0

    def e(self, s):
        self.lines.append(s)

    def label(self, stem):
        self.uid += 1
        return f"{stem}_{self.uid}_%="


# ---------------------------------------------------------------------------- building blocks
def mfma_qk(first, s_base, nt, frag, ks):
    d = V(s_base + 16 * nt, 16)
    c = V(NT[nt], 16) if first else d
    return f"v_mfma_f32_32x32x16_bf16 {d}, {V(FR + 4 * (frag % 8), 4)}, {A(128 + 4 * (8 * nt + ks), 4)}, {c}"


def mfma_pv(mt, nt, frag, p_base, kk):
    o = A(16 * (2 * mt + nt), 16)
    return f"v_mfma_f32_32x32x16_bf16 {o}, {V(FR + 4 * (frag % 8), 4)}, {V(p_base + 4 * (2 * nt + kk), 4)}, {o}"


def frag_source(R, par, f):
    """(address register, immediate) of operand fragment f of step (R, par)."""
    if f < 8:                                   # K fragment of step t+1
        if R < 3:
            return XOK + f, par * PAGE + (R + 1) * 8192
        return XOK + f, (1 - par) * PAGE        # first step of page q+1
    g = f - 8
    mt, kk = g & 3, g >> 2                      # an accumulator tile is revisited 8 MFMAs later
    if R == 0:                                  # V of the last step of page q-1
        return XOV + 6 + kk, (1 - par) * PAGE + mt * 8192
    return XOV + 2 * (R - 1) + kk, par * PAGE + mt * 8192


def ds_read_frag(f, src):
    reg, imm = src
    return f"ds_read_b128 {V(FR + 4 * (f % 8), 4)}, {V(reg)} offset:{imm}"


def tile_max_ops(s_base):
    """16 ops leaving max over the 16 accumulator registers of each column tile in MX[nt]."""
    ops = []
    for nt in range(2):
        b = s_base + 16 * nt
        m = V(MX[nt])
        ops.append(f"v_max3_f32 {m}, {V(b)}, {V(b + 1)}, {V(b + 2)}")
        for k in range(6):
            ops.append(f"v_max3_f32 {m}, {m}, {V(b + 3 + 2 * k)}, {V(b + 4 + 2 * k)}")
        ops.append(f"v_max_f32 {m}, {m}, {V(b + 15)}")
    return ops


def emit_page_address(E, which, advance):
    """Scalar part of a page request: move the (block, page) cursor of the K (which=0) or V
    (which=1) stream on by one page -- staying on the last visible page once the end is reached
    (the extra copies are never read) -- and leave the page's global address in s[S_ADDR:+1]."""
    kb, pg = (S_KKB, S_KPG) if which == 0 else (S_VKB, S_VPG)
    t = S_T
    if advance:
        E.e(f"s_add_u32 s{t}, s{pg}, 1")                         # pg + 1
        E.e(f"s_cmp_eq_u32 s{t}, s{S_P}")
        E.e(f"s_cselect_b32 s{t}, 0, s{t}")                      # wrapped page
        E.e(f"s_addc_u32 s{t + 1}, s{kb}, 0")                    # kb + (wrapped ? 1 : 0): scc still set by cmp
        E.e(f"s_cmp_lt_u32 s{t + 1}, s{S_NKVB}")                 # still inside the visible blocks?
        E.e(f"s_cselect_b32 s{pg}, s{t}, s{pg}")
        E.e(f"s_cselect_b32 s{kb}, s{t + 1}, s{kb}")
    # 64-bit byte offset: table[kb] + pg*stride + which*PAGE, then + pool base
    E.e(f"v_readlane_b32 s{t + 2}, {V(TBLLO)}, s{kb}")
    E.e(f"v_readlane_b32 s{t + 3}, {V(TBLHI)}, s{kb}")
    E.e(f"s_mul_i32 s{t + 4}, s{pg}, s{S_STRIDE}")
    E.e(f"s_mul_hi_u32 s{t + 5}, s{pg}, s{S_STRIDE}")
    E.e(f"s_add_u32 s{t + 2}, s{t + 2}, s{t + 4}")
    E.e(f"s_addc_u32 s{t + 3}, s{t + 3}, s{t + 5}")
    if which:
        E.e(f"s_add_u32 s{t + 2}, s{t + 2}, {PAGE}")
        E.e(f"s_addc_u32 s{t + 3}, s{t + 3}, 0")
    E.e(f"s_add_u32 s{S_ADDR}, s{S_POOL}, s{t + 2}")
    E.e(f"s_addc_u32 s{S_ADDR + 1}, s{S_POOL + 1}, s{t + 3}")


def emit_page_load(E, i, lds_slot_off):
    """Load number i (0..7) of the requested page: 64 lanes x 16 B -> 1 KB of LDS at
    slot + 4096 i + 1024 wave (M0 carries the LDS address, the VGPR the byte offset in the page)."""
    E.e(f"s_add_u32 m0, s{S_M0B}, {lds_slot_off + 4096 * i}")
    if not ABL & 4:
        E.e(f"global_load_lds_dwordx4 {V(DMAOFF + i)}, s[{S_ADDR}:{S_ADDR + 1}]")


def emit_issue_page(E, which, lds_slot_off, advance):
    emit_page_address(E, which, advance)
    for i in range(8):
        emit_page_load(E, i, lds_slot_off)


def emit_mask(E, s_base, valid_sreg):
    """Scores of keys at or past `valid` (keys of this 32-key step) become -inf, both column tiles."""
    E.e(f"v_mov_b32 {V(RT[0])}, 0xff800000")
    for i in range(16):
        const = 8 * (i >> 2) + (i & 3)
        E.e(f"s_sub_i32 s{S_T}, s{valid_sreg}, {const}")
        E.e(f"v_cmp_lt_i32 vcc, {V(KIDX)}, s{S_T}")                 # key row < valid
        for nt in range(2):
            r = V(s_base + 16 * nt + i)
            E.e(f"v_cndmask_b32 {r}, {V(RT[0])}, {r}, vcc")


def emit_settle(E, s_base, p_wait_base, first=False):
    """Reference update for the S tile at s_base (its maximum, relative to the current m_ref, is in
    MX): if some score exceeds m_ref by more than the slack, m_ref moves up to the row maximum and
    everything formed against the old reference is rescaled: row sums, accumulators, the P tile
    still waiting for its PV product, and this S tile itself.  first=True: unconditional (tile 0)."""
    cold, back = E.label("RARE"), E.label("BACK")
    if first:
        E.e(f"s_branch {cold}")
    else:
        E.e(f"v_cmp_lt_f32 vcc, 0x41000000, {V(MX[0])}")           # 8.0 < max
        E.e(f"s_mov_b64 s[{S_VCC}:{S_VCC + 1}], vcc")
        E.e(f"v_cmp_lt_f32 vcc, 0x41000000, {V(MX[1])}")
        E.e(f"s_or_b64 vcc, vcc, s[{S_VCC}:{S_VCC + 1}]")
        E.e(f"s_cbranch_vccnz {cold}")
    E.e(f"{back}:")
    c = E.cold
    c.append(f"{cold}:")
    c.append("s_nop 15\ns_nop 15\ns_nop 15")            # every MFMA issued so far has written back
    for nt in range(2):
        t, other, delta, alpha = V(MX[nt]), V(RT[3]), V(RT[4]), V(RT[6])
        c.append(f"ds_bpermute_b32 {other}, {V(XLANE)}, {t}")        # the partner lane's (lane ^ 32) maximum
        c.append("s_waitcnt lgkmcnt(0)")
        c.append(f"v_max_f32 {delta}, {t}, {other}")
        if not first:
            c.append(f"v_max_f32 {delta}, 0, {delta}")               # the reference never moves down
        c.append(f"v_exp_f32_e64 {alpha}, -{delta}")
        c.append("s_nop 3")                              # a trans result is not forwarded to the next VALU op
        for k in range(2):
            c.append(f"v_mul_f32 {V(LACC + 2 * nt + k)}, {V(LACC + 2 * nt + k)}, {alpha}")
        for mt in range(4):
            for i in range(16):
                acc = A(16 * (2 * mt + nt) + i)
                tmp = V(RT[8 + (i % 8)])
                c.append(f"v_accvgpr_read_b32 {tmp}, {acc}")
                c.append(f"v_mul_f32 {tmp}, {tmp}, {alpha}")
                c.append(f"v_accvgpr_write_b32 {acc}, {tmp}")
        for kk in range(2):
            for w in range(4):
                r = V(p_wait_base + 4 * (2 * nt + kk) + w)
                lo, hi = V(RT[8]), V(RT[9])
                c.append(f"v_lshlrev_b32 {lo}, 16, {r}")
                c.append(f"v_and_b32 {hi}, 0xffff0000, {r}")
                c.append(f"v_mul_f32 {lo}, {lo}, {alpha}")
                c.append(f"v_mul_f32 {hi}, {hi}, {alpha}")
                c.append(f"v_cvt_pk_bf16_f32 {r}, {lo}, {hi}")
        for i in range(16):                              # -m_ref operand and the tile itself
            c.append(f"v_sub_f32 {V(NT[nt] + i)}, {V(NT[nt] + i)}, {delta}")
            c.append(f"v_sub_f32 {V(s_base + 16 * nt + i)}, {V(s_base + 16 * nt + i)}, {delta}")
    c.append("s_nop 7")
    c.append(f"s_branch {back}")


def emit_mask_check(E, s_base, pg_sreg, sub):
    """If the tile at s_base is the ragged tail of a block's last page: mask it and redo its max."""
    cold, back = E.label("MASK"), E.label("MBACK")
    E.e(f"s_cmp_eq_u32 s{pg_sreg}, s{S_PM1}")
    E.e(f"s_cselect_b32 s{S_T + 8}, s{S_VLAST + sub}, 32")
    E.e(f"s_cmp_lt_u32 s{S_T + 8}, 32")
    E.e(f"s_cbranch_scc1 {cold}")
    E.e(f"{back}:")
    sub_e = Emitter()
    emit_mask(sub_e, s_base, S_T + 8)
    E.cold.append(f"{cold}:")
    E.cold.append("s_nop 15\ns_nop 15\ns_nop 15")
    E.cold.extend(sub_e.lines)
    E.cold.extend(tile_max_ops(s_base))
    E.cold.append(f"s_branch {back}")


def p_word(p_base, j):
    """VGPR of the packed pair that ends at element j (odd) of the tile being exponentiated."""
    nt, e = j >> 4, j & 15
    return p_base + 4 * (2 * nt + (e >> 3)) + ((e & 7) >> 1)


def emit_pack(E, j, p_cur):
    """elements j-1, j -> one bf16 pair of P^T (round to nearest even)."""
    E.e(f"v_cvt_pk_bf16_f32 {V(p_word(p_cur, j))}, {V(PX[(j - 1) & 3])}, {V(PX[j & 3])}")


def emit_rowsum(E, j, p_cur):
    """row sums += the two (unrounded) probabilities of the pair ending at element j: one
    accumulator for even, one for odd elements of each column tile.  (A v_dot2_f32_bf16 on the packed
    pair would halve the instruction count but measured 2.3 ms slower per forward.)"""
    nt = j >> 4
    E.e(f"v_add_f32 {V(LACC + 2 * nt)}, {V(LACC + 2 * nt)}, {V(PX[(j - 1) & 3])}")
    E.e(f"v_add_f32 {V(LACC + 2 * nt + 1)}, {V(LACC + 2 * nt + 1)}, {V(PX[j & 3])}")


def exp_slot(e):
    """Issue slot of the exponential of element e (0..31) of the tile: two each in slots 0 and 1,
    then one per slot, so that the last one issues in slot 29 and everything derived from it
    (pack, row sum) still fits under the step's last MFMAs."""
    return e >> 1 if e < 4 else e - 2


def emit_step(E, R, par):
    cur, nxt = ("A", "B") if R % 2 == 0 else ("B", "A")
    s_cur, s_next = S_TILE[cur], S_TILE[nxt]
    p_prev, p_cur = (P_TILE["B"], P_TILE["A"]) if R % 2 == 0 else (P_TILE["A"], P_TILE["B"])
    nR, npar = ((R + 1) & 3, par if R < 3 else 1 - par)
    max_ops = tile_max_ops(s_next)
    max_at = {}                                           # slot -> ops (slots 18..29: QK retired)
    for k, op in enumerate(max_ops):
        max_at.setdefault(18 + (k * 12) // 16, []).append(op)
    exps_at, packs_at = {}, {}
    for e in range(32):
        exps_at.setdefault(exp_slot(e), []).append(e)
        if e & 1:                                         # a trans result is consumed >= 2 slots later
            packs_at.setdefault(exp_slot(e) + 2, []).append(e)
    px_holds = {}                                         # PX register -> element, to check the ring

    E.e(f"; ---- step R={R} parity={par}")
    for i in range(32):
        f, nt = i >> 1, i & 1
        if R == 1 and i == 0:                             # V(q) visible; slot of V(q-1) free -> V(q+1)
            E.e("s_waitcnt vmcnt(8)")
            if not ABL & 8:
                E.e("s_barrier")
            emit_page_address(E, 1, advance=True)
        if R == 2 and i == 24:                            # K(q+1) visible; slot of K(q) free -> K(q+2)
            E.e("s_waitcnt vmcnt(8)")
            if not ABL & 8:
                E.e("s_barrier")
            emit_page_address(E, 0, advance=True)
        if nt == 0 and not ABL & 2:
            E.e(f"s_waitcnt lgkmcnt({D_AHEAD - 1})")      # fragment f has landed
        if f < 8:
            E.e(mfma_qk(f == 0, s_next, nt, f, f))
        else:
            g = f - 8
            E.e(mfma_pv(g & 3, nt, f, p_prev, g >> 2))
        # fillers: page load, operand prefetch, softmax of s_cur, running max of s_next
        if R == 1 and i < 8:
            emit_page_load(E, i, VRING + (1 - par) * PAGE)
        if R == 2 and i >= 24:
            emit_page_load(E, i - 24, par * PAGE)
        if nt == 0 and not ABL & 2:
            fa = f + D_AHEAD
            if fa < 16:
                E.e(ds_read_frag(fa, frag_source(R, par, fa)))
            else:
                E.e(ds_read_frag(fa - 16, frag_source(nR, npar, fa - 16)))
        if ABL & 1:
            continue
        for j in packs_at.get(i, []):
            assert px_holds[PX[(j - 1) & 3]] == j - 1 and px_holds[PX[j & 3]] == j
            emit_pack(E, j, p_cur)
            emit_rowsum(E, j, p_cur)
        for e in exps_at.get(i, []):
            px_holds[PX[e & 3]] = e
            E.e(f"v_exp_f32 {V(PX[e & 3])}, {V(s_cur + 16 * (e >> 4) + (e & 15))}")
        for op in max_at.get(i, []):
            E.e(op)
        # the tile just produced is exponentiated in the next step: mask its ragged tail (slot 30),
        # then settle the exponent reference (after the last MFMA)
        if i == 30:
            if R < 3:
                emit_mask_check(E, s_next, S_PGCUR, R + 1)
            else:
                emit_mask_check(E, s_next, S_PGNEXT, 0)
    if ABL & 1:
        return
    emit_settle(E, s_next, p_cur)


def emit_page_end(E):
    """Per-page scalar bookkeeping: page-in-block counters of pages q and q+1."""
    E.e(f"s_mov_b32 s{S_PGCUR}, s{S_PGNEXT}")
    E.e(f"s_add_u32 s{S_T}, s{S_PGNEXT}, 1")
    E.e(f"s_cmp_eq_u32 s{S_T}, s{S_P}")
    E.e(f"s_cselect_b32 s{S_PGNEXT}, 0, s{S_T}")


def emit_drain(E, par_last):
    """PV of the final step: V page (parity par_last), keys 96..127, P tile B."""
    for g in range(8):
        mt, kk = g & 3, g >> 2
        E.e(f"ds_read_b128 {V(FR + 4 * g, 4)}, {V(XOV + 6 + kk)} offset:{par_last * PAGE + mt * 8192}")
    E.e("s_waitcnt lgkmcnt(0)")
    for g in range(8):
        for nt in range(2):
            E.e(mfma_pv(g & 3, nt, g, P_TILE["B"], g >> 2))


def generate():
    E = Emitter()
    # ---- set-up: inputs to fixed registers
    E.e(f"s_mov_b32 s{S_NLEFT}, %[n_pages]")
    E.e(f"s_mov_b32 s{S_P}, %[ppb]")
    E.e(f"s_sub_u32 s{S_PM1}, s{S_P}, 1")
    E.e(f"s_mov_b32 s{S_STRIDE}, %[stride]")
    E.e(f"s_mov_b32 s{S_NKVB}, %[n_kvb]")
    E.e(f"s_mov_b64 s[{S_POOL}:{S_POOL + 1}], %[pool]")
    E.e(f"s_mov_b32 s{S_LDS0}, %[lds0]")
    E.e(f"s_lshl_b32 s{S_M0B}, %[wave], 10")
    E.e(f"s_add_u32 s{S_M0B}, s{S_M0B}, s{S_LDS0}")
    E.e(f"s_mov_b32 s{S_LASTV}, %[last_valid]")
    for sub in range(4):                                  # clamp(last_valid - 32*sub, 0, 32)
        E.e(f"s_sub_i32 s{S_VLAST + sub}, s{S_LASTV}, {32 * sub}")
        E.e(f"s_max_i32 s{S_VLAST + sub}, s{S_VLAST + sub}, 0")
        E.e(f"s_min_i32 s{S_VLAST + sub}, s{S_VLAST + sub}, 32")
    for i in range(8):
        E.e(f"v_add_u32 {V(DMAOFF + i)}, {4096 * i}, %[lane_off]")
    E.e(f"v_mov_b32 {V(TBLLO)}, %[tbl_lo]")
    E.e(f"v_mov_b32 {V(TBLHI)}, %[tbl_hi]")
    E.e(f"v_mov_b32 {V(KIDX)}, %[kidx]")
    E.e(f"v_mov_b32 {V(XLANE)}, %[xlane]")
    for j in range(8):
        E.e(f"v_xor_b32 {V(XOK + j)}, {j << 5}, %[xo0]")
        E.e(f"v_add_u32 {V(XOK + j)}, s{S_LDS0}, {V(XOK + j)}")
        E.e(f"v_add_u32 {V(XOV + j)}, {VRING}, {V(XOK + j)}")
    for r in range(128):
        E.e(f"v_accvgpr_write_b32 {A(r)}, 0")
    for r in range(4):
        E.e(f"v_mov_b32 {V(LACC + r)}, 0")
    for nt in range(2):                                   # m_ref = 0 until tile 0 has been seen
        for i in range(16):
            E.e(f"v_mov_b32 {V(NT[nt] + i)}, 0")
    for r in range(16):
        E.e(f"v_mov_b32 {V(P_TILE['B'] + r)}, 0")
    # the walk starts at page pg0 of visible block kb0 (0, 0 unless the KV range of a tile is split)
    E.e(f"s_mov_b32 s{S_PGCUR}, %[pg0]")
    E.e(f"s_add_u32 s{S_T}, s{S_PGCUR}, 1")
    E.e(f"s_cmp_eq_u32 s{S_T}, s{S_P}")
    E.e(f"s_cselect_b32 s{S_PGNEXT}, 0, s{S_T}")
    for r in (S_KKB, S_VKB):
        E.e(f"s_mov_b32 s{r}, %[kb0]")
    for r in (S_KPG, S_VPG):
        E.e(f"s_mov_b32 s{r}, %[pg0]")
    # ---- K(0), V(0), K(1) in flight; wait for the first two, publish
    emit_issue_page(E, 0, 0, advance=False)
    emit_issue_page(E, 1, VRING, advance=False)
    emit_issue_page(E, 0, PAGE, advance=True)
    E.e("s_waitcnt vmcnt(8) lgkmcnt(0)")
    E.e("s_barrier")
    # ---- S tile of step 0 into tile A, its mask, max and reference
    for f in range(8):
        E.e(f"ds_read_b128 {V(FR + 4 * f, 4)}, {V(XOK + f)} offset:0")
    E.e("s_waitcnt lgkmcnt(0)")
    for f in range(8):
        for nt in range(2):
            E.e(mfma_qk(f == 0, S_TILE["A"], nt, f, f))
    E.e("s_nop 15\ns_nop 15\ns_nop 15")
    for op in tile_max_ops(S_TILE["A"]):
        E.e(op)
    emit_mask_check(E, S_TILE["A"], S_PGCUR, 0)
    emit_settle(E, S_TILE["A"], P_TILE["B"], first=True)
    # first operand fragments of step (R=0, parity 0)
    for f in range(D_AHEAD):
        E.e(ds_read_frag(f, frag_source(0, 0, f)))

    # ---- main loop, two pages per trip (ring parity is compile-time)
    loop, exit_even, exit_odd, done = (E.label("LOOP"), E.label("EXIT_EVEN"), E.label("EXIT_ODD"),
                                        E.label("DONE"))
    E.e(f"{loop}:")
    for par in range(2):
        for R in range(4):
            emit_step(E, R, par)
        emit_page_end(E)
        E.e(f"s_sub_u32 s{S_NLEFT}, s{S_NLEFT}, 1")
        E.e(f"s_cmp_eq_u32 s{S_NLEFT}, 0")
        E.e(f"s_cbranch_scc1 {exit_even if par == 0 else exit_odd}")
    E.e(f"s_branch {loop}")
    E.e(f"{exit_even}:")
    E.e("s_waitcnt lgkmcnt(0)")
    emit_drain(E, 0)
    E.e(f"s_branch {done}")
    E.e(f"{exit_odd}:")
    E.e("s_waitcnt lgkmcnt(0)")
    emit_drain(E, 1)
    E.e(f"s_branch {done}")
    # ---- out-of-line blocks
    for ln in E.cold:
        E.e(ln)
    E.e(f"{done}:")
    E.e("s_waitcnt vmcnt(0)")                              # trailing (unused) page loads have landed
    E.e("s_nop 15\ns_nop 15\ns_nop 15")                    # the last MFMAs have written back
    for r in range(128):                                   # results leave in v[0:127]
        E.e(f"v_accvgpr_read_b32 {V(r)}, {A(r)}")
    return E.lines


def main(out_path):
    lines = generate()
    text = []
    for ln in lines:
        for part in ln.split("\n"):
            text.append(part)
    with open(out_path, "w") as f:
        f.write("// Generated by gen_attn_core.py -- do not edit.\n")
        for t in text:
            f.write('"' + t.replace("\\", "\\\\").replace('"', '\\"') + '\\n"\n')
    # registers the block uses beyond its operands (v148..v151 are outputs)
    clob = [f"v{i}" for i in range(128, 224) if not 148 <= i <= 151 and i not in (184, 200)] + [f"a{i}" for i in range(0, 128)] + [f"s{i}" for i in range(36, 96)]
    clob_path = out_path.replace("attn_core_gfx950.inc", "attn_core_clobbers.inc")
    with open(clob_path, "w") as f:
        f.write("// Generated by gen_attn_core.py -- do not edit.\n#define CA_CORE_CLOBBERS \\\n")
        for i in range(0, len(clob), 12):
            chunk = ", ".join(f'"{c}"' for c in clob[i:i + 12])
            f.write("  " + chunk + (", \\\n" if i + 12 < len(clob) else "\n"))
    print(f"{out_path}: {len(text)} lines")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "attn_core_gfx950.inc")
