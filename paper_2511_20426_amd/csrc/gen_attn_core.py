#!/usr/bin/env python3
"""Emits attn_core_gfx950.inc: the hand-scheduled main loop of the bf16 cascaded-attention kernel.

The loop is written as one inline-assembly block (included by attn_bf16.hip) because its speed
rests on two things a compiler will not hold still for:

  * issue order -- a wave issues in order, one instruction per 4 cycles, and an MFMA occupies the
    matrix pipe for 32 cycles: between two MFMAs there is room for exactly 6 more issue quanta
    (see "issue-slot scheduling" below), and the softmax of the previous tile, the operand
    prefetch and the page traffic have to be dealt out so that no slot holds more;
  * register files -- Q fragments and the O^T accumulators live in AGPRs, which VALU code never
    touches in the loop; S^T tiles, P^T and the K/V operand fragments live in VGPRs.

Pipeline (a "step" is 32 keys, a page is 4 steps; t counts steps):
    QK(t+1): 16 MFMAs  S_next = K_frag x Q                      (K fragments from LDS)
    SM(t)  : p = exp2(S_cur), bf16 pack, row sums                (VALU; S_cur already holds
             s*c - m_ref: Q is pre-scaled by c = log2(e)/sqrt(D) and QK starts from -m_ref)
    PV(t-1): 16 MFMAs  O^T   += V_frag x P_prev                  (V fragments from LDS)
The three are independent inside a step.  K and V pages stream global -> LDS (no registers) into
two 2-page rings; per page there is one barrier that publishes V(q) and frees V(q-1)'s slot
(before step 1) and one that publishes K(q+1) and frees K(q)'s slot (in step 2).

The exponent reference m_ref of a row is lazy: it starts as the maximum of the row's first tile
and moves only when it has to.  No maximum is taken in the loop; instead the 16 probabilities a
lane forms in a step are summed on their own, and a sum above 2^16 (or inf: exp2 against a stale
reference may overflow) sends the wave to an out-of-line block at the end of the step, which
takes the tile's maximum, forms the step's probabilities again from the S tile (still in
registers) against the raised reference and rescales what earlier steps left.  The same branch
serves the rare step whose S tile needs its ragged tail masked.

Register map (fixed):
  a[0:127]    O^T accumulators, tile (mt, nt) at a[16*(2*mt+nt) ..]
  a[128:191]  Q fragments, (nt, ks) at a[128 + 4*(8*nt+ks) ..]
  v[0:31]     S tile A (nt 0: v0.., nt 1: v16..)     v[32:63]  S tile B
  v[64:79]    P^T tile A, (nt, kk) at v[64 + 4*(2*nt+kk) ..]      v[80:95]  P^T tile B
  v[96:127]   ring of 8 operand fragments
  v[128:135]  LDS address of chunk pair j in the K ring, v[136:143] the same in the V ring
  v148, v150  running row sums of column tile 0 / 1 (v149, v151 stay zero)
  v152, v153  row sums of the current step, column tile 0 / 1
  v158..v175  temporaries of the out-of-line blocks
  v[184:199], v[200:215]  -m_ref of column tile 0 / 1, replicated 16 times: the C operand of the
              first MFMA of every S tile, so a tile comes out of the matrix pipe as s*c - m_ref
  v[216:223]  lane's byte offset inside a page for page load i = 0..7
  v[224:255]  the 32 probabilities of the step before they are packed
  v177,v178   address of page 0 of each KV block for this head (lane i = block i), low / high word
  v179        4*(lane/32): first key row this lane holds in a 32x32 accumulator
  v180        4*(lane ^ 32): ds_bpermute address of the lane holding the other half of this row
"""
from __future__ import annotations

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from issue_sched import Atom, quanta, schedule  # noqa: E402

D_AHEAD = 5          # operand fragments are read this many MFMA pairs ahead of use
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
TS = [152, 153]      # row sums of the current step, per column tile
MX = [158, 159]
PX = 224             # 224..255: the 32 probabilities of the step, before packing
RT = list(range(160, 176))     # rare-path temporaries
TBLLO, TBLHI, KIDX, XLANE = 177, 178, 179, 180
DMAOFF = 216         # 216..223: lane's byte offset in a page for load i (+4096 i)

# scalar registers (all inside the clobbered range s36..s95)
S_NLEFT, S_P, S_PM1, S_STRIDE, S_NKVB = 41, 42, 43, 44, 45
S_M0B, S_LASTV = 48, 49
S_VLAST = 50         # 50..53
S_PGCUR, S_PGNEXT = 54, 55
S_KKB, S_KPG = 56, 57  # page cursor: visible KV block, page in it
S_T = 60             # 60..69 temporaries
S_ADDR = 70          # 70,71
S_LDS0 = 74
S_ADDRV = 76         # 76,77
S_RG = 78            # 78,79: nonzero if the tile just produced needs its tail masked
S_VLP = 80           # 80..87: per 32-key step of a page, (-1 if a block's last page is ragged there, 0)


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


def page_advance_lines():
    """Moves the page cursor (kb, pg) on by one page -- staying on the last visible page once the
    end is reached (the extra copies are never read) -- and leaves the K page's global address in
    s[S_ADDR:+1]; the V page of the same pair is PAGE bytes further.  Returned as groups of lines
    that must stay contiguous (each group hands a condition over in SCC)."""
    kb, pg, t = S_KKB, S_KPG, S_T
    return [
        [f"s_add_u32 s{t}, s{pg}, 1", f"s_cmp_eq_u32 s{t}, s{S_P}", f"s_cselect_b32 s{t}, 0, s{t}",
         f"s_addc_u32 s{t + 1}, s{kb}, 0"],                      # kb + (wrapped ? 1 : 0): scc from the cmp
        [f"s_cmp_lt_u32 s{t + 1}, s{S_NKVB}", f"s_cselect_b32 s{pg}, s{t}, s{pg}",
         f"s_cselect_b32 s{kb}, s{t + 1}, s{kb}"],
    ] + page_address_lines()


def page_address_lines():
    kb, pg, t = S_KKB, S_KPG, S_T
    return [
        [f"v_readlane_b32 s{t + 2}, {V(TBLLO)}, s{kb}"],
        [f"v_readlane_b32 s{t + 3}, {V(TBLHI)}, s{kb}"],
        [f"s_mul_i32 s{t + 4}, s{pg}, s{S_STRIDE}"],
        [f"s_mul_hi_u32 s{t + 5}, s{pg}, s{S_STRIDE}"],
        [f"s_add_u32 s{S_ADDR}, s{t + 2}, s{t + 4}", f"s_addc_u32 s{S_ADDR + 1}, s{t + 3}, s{t + 5}"],
    ]


def v_address_lines():
    """V page of the pair whose K address is in s[S_ADDR:+1]."""
    return [[f"s_add_u32 s{S_ADDRV}, s{S_ADDR}, {PAGE}", f"s_addc_u32 s{S_ADDRV + 1}, s{S_ADDR + 1}, 0"]]


def page_load_lines(i, lds_slot_off, which):
    """Load number i (0..7) of a page: 64 lanes x 16 B -> 1 KB of LDS at slot + 4096 i + 1024 wave
    (M0 carries the LDS address, the VGPR the byte offset in the page)."""
    a = S_ADDRV if which else S_ADDR
    return [f"s_add_u32 m0, s{S_M0B}, {lds_slot_off + 4096 * i}",
            f"global_load_lds_dwordx4 {V(DMAOFF + i)}, s[{a}:{a + 1}]"]


def emit_issue_page(E, which, lds_slot_off):
    for i in range(8):
        for ln in page_load_lines(i, lds_slot_off, which):
            E.e(ln)


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


def emit_first_reference(E, s_base):
    """The exponent reference of a row starts as the maximum of its first tile (at s_base, its
    per-lane maxima in MX): the tile and the -m_ref operand move by it.  Nothing has been
    accumulated yet, so there is nothing to rescale."""
    E.e("s_nop 15\ns_nop 15\ns_nop 15")                   # every MFMA issued so far has written back
    for nt in range(2):
        t, other, delta = V(MX[nt]), V(RT[3]), V(RT[4])
        E.e(f"ds_bpermute_b32 {other}, {V(XLANE)}, {t}")             # the partner lane's (lane ^ 32) maximum
        E.e("s_waitcnt lgkmcnt(0)")
        E.e(f"v_max_f32 {delta}, {t}, {other}")
        for i in range(16):
            E.e(f"v_sub_f32 {V(NT[nt] + i)}, {V(NT[nt] + i)}, {delta}")
            E.e(f"v_sub_f32 {V(s_base + 16 * nt + i)}, {V(s_base + 16 * nt + i)}, {delta}")


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


# ---------------------------------------------------------------------------- issue-slot scheduling
# (model and scheduler: issue_sched.py)
CAP = 8.2            # issue quanta per MFMA slot the scheduler may fill (8 = the slot; a little over pays)


E_SPREAD = 22        # the 32 exponentials of a step are due by this slot
THRESH = "0x47800000"     # 2^16: a step's row sum of 16 probabilities above this moves the reference
K_BARRIER_SLOT = 16  # step 2: K(q+1) visible, slot of K(q) free
N_KLOADS_R2 = 2      # of the 8 loads of K(q+2), how many issue in step 2 (the rest in step 3)


def build_step(R, par):
    """One 32-key step as a list of 32 slots: (MFMA line, [lines issued after it])."""
    cur, nxt = ("A", "B") if R % 2 == 0 else ("B", "A")
    s_cur, s_next = S_TILE[cur], S_TILE[nxt]
    p_prev, p_cur = (P_TILE["B"], P_TILE["A"]) if R % 2 == 0 else (P_TILE["A"], P_TILE["B"])
    nR, npar = ((R + 1) & 3, par if R < 3 else 1 - par)
    cold, back = f"COLD_{R}_{par}_%=", f"BACK_{R}_{par}_%="

    mfma, head, tail = [None] * 32, [[] for _ in range(32)], [[] for _ in range(32)]
    for i in range(32):
        f, nt = i >> 1, i & 1
        if f < 8:
            mfma[i] = mfma_qk(f == 0, s_next, nt, f, f)
        else:
            g = f - 8
            mfma[i] = mfma_pv(g & 3, nt, f, p_prev, g >> 2)
        if nt == 0:                                        # operand prefetch, D_AHEAD pairs ahead
            fa = f + D_AHEAD
            src = frag_source(R, par, fa) if fa < 16 else frag_source(nR, npar, fa - 16)
            head[i].append(ds_read_frag(fa % 16, src))
        # what must precede the next MFMA: every other pair waits for its two fragments
        if (i + 1) % 4 == 0:
            tail[i].append(f"s_waitcnt lgkmcnt({D_AHEAD - 2})")
    if R == 0:                                             # before step 1: V(q) visible, V(q-1)'s slot free
        tail[31] += ["s_waitcnt vmcnt(@VMCNT_V@)", "s_barrier"]
    if R == 2:
        tail[K_BARRIER_SLOT - 1] += ["s_waitcnt vmcnt(@VMCNT_K@)", "s_barrier"]

    atoms = []
    # row sums of the previous step join the running sums; this step's start afresh
    lacc = [Atom([f"v_add_f32 {V(LACC + 2 * nt)}, {V(LACC + 2 * nt)}, {V(TS[nt])}"], 0, 0, hard=1) for nt in range(2)]
    atoms += lacc
    exps = [Atom([f"v_exp_f32 {V(PX + e)}, {V(s_cur + e)}"], 0, (e * E_SPREAD) // 32, hard=min(E_SPREAD + 4, 27)) for e in range(32)]
    atoms += exps
    last_sum = [None, None]
    for j in range(1, 32, 2):
        nt = j >> 4
        deps, dl = [exps[j - 1], exps[j]], (j * E_SPREAD) // 32 + 5
        atoms.append(Atom([f"v_cvt_pk_bf16_f32 {V(p_word(p_cur, j))}, {V(PX + j - 1)}, {V(PX + j)}"],
                          0, dl, deps, 2, hard=29))
        if last_sum[nt] is None:
            sm = [Atom([f"v_add_f32 {V(TS[nt])}, {V(PX + j - 1)}, {V(PX + j)}"], 0, dl, deps, 2, hard=28)]
            sm[0].after.append((lacc[nt], 0))
        else:
            sm = [Atom([f"v_add_f32 {V(TS[nt])}, {V(TS[nt])}, {V(PX + k)}"], 0, dl, deps, 2, hard=28)
                  for k in (j - 1, j)]
            sm[0].after.append((last_sum[nt], 0))
            sm[1].after.append((sm[0], 0))
        atoms += sm
        last_sum[nt] = sm[-1]
    # is the tile just produced the ragged tail of a block's last page?
    pg, sub = (S_PGCUR, R + 1) if R < 3 else (S_PGNEXT, 0)
    rag = Atom([f"s_cmp_eq_u32 s{pg}, s{S_PM1}",
                f"s_cselect_b64 s[{S_RG}:{S_RG + 1}], s[{S_VLP + 2 * sub}:{S_VLP + 2 * sub + 1}], 0"], 0, 6, hard=24)
    det = Atom([f"v_max_f32 {V(RT[1])}, {V(TS[0])}, {V(TS[1])}",
                f"v_cmp_lt_f32 vcc, {THRESH}, {V(RT[1])}"], 0, 28, [last_sum[0], last_sum[1]], 0, hard=29)
    # scc travels from here to the branch after the last MFMA: nothing that writes scc may
    # issue in slots 30 and 31 (every such atom has hard <= 29)
    orr = Atom([f"s_or_b64 s[{S_T + 8}:{S_T + 9}], vcc, s[{S_RG}:{S_RG + 1}]"], 30, 30, [det, rag], 1, hard=30)
    atoms += [rag, det, orr]
    tail[31].insert(0, f"{back}:")
    tail[31].insert(0, f"s_cbranch_scc1 {cold}")
    # page traffic
    loads = []
    if R == 0:                                             # address of V(q+1), then of K(q+2)
        prev = None
        for k, grp in enumerate(v_address_lines() + page_advance_lines()):
            prev = Atom(grp, 2, 6 + 3 * k, [prev] if prev else [], 0, hard=29)
            atoms.append(prev)
    if R == 1:                                             # V(q+1) into the slot V(q-1) left
        for i in range(8):
            loads.append(Atom(page_load_lines(i, VRING + (1 - par) * PAGE, 1), 0, 2 + 4 * i, tag=("load", 1), hard=29))
    if R == 2:                                             # K(q+2) into the slot K(q) left
        for i in range(N_KLOADS_R2):
            loads.append(Atom(page_load_lines(i, par * PAGE, 0), K_BARRIER_SLOT,
                              K_BARRIER_SLOT + 2 + (i * (26 - K_BARRIER_SLOT)) // N_KLOADS_R2, tag=("load", 0), hard=29))
    if R == 3:
        n = 8 - N_KLOADS_R2
        for i in range(n):
            loads.append(Atom(page_load_lines(N_KLOADS_R2 + i, par * PAGE, 0), 0, 2 + (i * 28) // n, tag=("load", 0), hard=29))
        # page-in-block counters of pages q and q+1 move on; one page less to go
        pe = Atom([f"s_mov_b32 s{S_PGCUR}, s{S_PGNEXT}", f"s_add_u32 s{S_T}, s{S_PGNEXT}, 1",
                   f"s_cmp_eq_u32 s{S_T}, s{S_P}", f"s_cselect_b32 s{S_PGNEXT}, 0, s{S_T}",
                   f"s_sub_u32 s{S_NLEFT}, s{S_NLEFT}, 1"], 0, 20, [rag], 1, hard=29)
        atoms.append(pe)
    atoms += loads

    fixed = [2.0 + sum(quanta(l) for l in head[i] + tail[i]) for i in range(32)]
    placed = schedule(fixed, atoms, CAP)
    for i in (30, 31):
        for a in placed[i]:
            assert not any(l.split()[0].startswith(("s_add", "s_sub", "s_cmp", "s_and", "s_mul")) for l in a.lines), a.lines
    slots = []
    for i in range(32):
        lines = list(head[i])
        for a in placed[i]:
            lines += a.lines
        lines += tail[i]
        slots.append((mfma[i], lines))
    return slots, (s_cur, s_next, p_cur, cold, back, (S_VLAST + (R + 1 if R < 3 else 0)))


def emit_cold(E, s_cur, s_next, p_cur, cold, back, valid_sreg):
    """Out-of-line end of a step, entered when some lane's row sum of the step crossed THRESH
    (vcc) or the tile just produced needs its ragged tail masked (s[S_RG]).

    Moving the reference: the probabilities of the step were formed against a reference that
    turned out too low (they may even have overflowed), so they are formed again from the S tile,
    which is still in registers: the row maximum relative to the old reference gives the shift
    delta >= 0; row sums and accumulators (all from earlier steps) are scaled by 2^-delta, the
    tile just produced and the -m_ref operand move by delta."""
    c = E.cold
    skip_ovf, done = E.label("NOOVF"), E.label("CDONE")
    c.append(f"{cold}:")
    c.append("s_nop 15\ns_nop 15\ns_nop 15")            # every MFMA issued so far has written back
    c.append(f"s_cbranch_vccz {skip_ovf}")
    for nt in range(2):
        b = s_cur + 16 * nt
        m, other, delta, alpha = V(MX[nt]), V(RT[3]), V(RT[4]), V(RT[6])
        c.append(f"v_max3_f32 {m}, {V(b)}, {V(b + 1)}, {V(b + 2)}")
        for k in range(6):
            c.append(f"v_max3_f32 {m}, {m}, {V(b + 3 + 2 * k)}, {V(b + 4 + 2 * k)}")
        c.append(f"v_max_f32 {m}, {m}, {V(b + 15)}")
        c.append(f"ds_bpermute_b32 {other}, {V(XLANE)}, {m}")       # the partner lane's (lane ^ 32) maximum
        c.append("s_waitcnt lgkmcnt(0)")
        c.append(f"v_max_f32 {delta}, {m}, {other}")
        c.append(f"v_max_f32 {delta}, 0, {delta}")                  # the reference never moves down
        c.append(f"v_exp_f32_e64 {alpha}, -{delta}")
        c.append("s_nop 3")                              # a trans result is not forwarded to the next VALU op
        c.append(f"v_mul_f32 {V(LACC + 2 * nt)}, {V(LACC + 2 * nt)}, {alpha}")
        for mt in range(4):
            for i in range(16):
                acc = A(16 * (2 * mt + nt) + i)
                tmp = V(RT[8 + (i % 8)])
                c.append(f"v_accvgpr_read_b32 {tmp}, {acc}")
                c.append(f"v_mul_f32 {tmp}, {tmp}, {alpha}")
                c.append(f"v_accvgpr_write_b32 {acc}, {tmp}")
        for i in range(16):                              # the step's probabilities again
            c.append(f"v_sub_f32 {V(b + i)}, {V(b + i)}, {delta}")
        for i in range(16):
            c.append(f"v_exp_f32 {V(PX + 16 * nt + i)}, {V(b + i)}")
        c.append("s_nop 3")
        c.append(f"v_add_f32 {V(TS[nt])}, {V(PX + 16 * nt)}, {V(PX + 16 * nt + 1)}")
        for i in range(2, 16):
            c.append(f"v_add_f32 {V(TS[nt])}, {V(TS[nt])}, {V(PX + 16 * nt + i)}")
        for j in range(16 * nt + 1, 16 * nt + 16, 2):
            c.append(f"v_cvt_pk_bf16_f32 {V(p_word(p_cur, j))}, {V(PX + j - 1)}, {V(PX + j)}")
        for i in range(16):                              # -m_ref operand and the tile just produced
            c.append(f"v_sub_f32 {V(NT[nt] + i)}, {V(NT[nt] + i)}, {delta}")
            c.append(f"v_sub_f32 {V(s_next + 16 * nt + i)}, {V(s_next + 16 * nt + i)}, {delta}")
    c.append(f"{skip_ovf}:")
    c.append(f"s_cmp_eq_u32 s{S_RG}, 0")
    c.append(f"s_cbranch_scc1 {done}")
    sub_e = Emitter()
    emit_mask(sub_e, s_next, valid_sreg)
    c.extend(sub_e.lines)
    c.append(f"{done}:")
    c.append("s_nop 7")
    c.append(f"s_branch {back}")


def emit_step(E, R, par, vmcnt):
    slots, cold_args = build_step(R, par)
    E.e(f"; ---- step R={R} parity={par}")
    for m, lines in slots:
        E.e(m)
        for ln in lines:
            E.e(ln.replace("@VMCNT_V@", str(vmcnt[0])).replace("@VMCNT_K@", str(vmcnt[1])))
    emit_cold(E, *cold_args)


def wait_counts():
    """vmcnt operands of the two page barriers: loads complete in issue order, so waiting for
    page X means allowing as many loads in flight as are issued after X's last one."""
    order = []                                            # (R, slot, stream) of every load of one page period
    for R in range(4):
        slots, _ = build_step(R, 0)
        for i, (_, lines) in enumerate(slots):
            for ln in lines:
                if ln.startswith("s_add_u32 m0"):
                    order.append((R, i, 1 if R == 1 else 0))
    assert len(order) == 16, order
    def after_last(stream, until):
        """loads issued after the last `stream` load of the previous page, up to time `until` of this page"""
        last = max(k for k, o in enumerate(order) if o[2] == stream)
        n_prev = len(order) - 1 - last
        n_now = sum(1 for o in order if (o[0], o[1]) <= until)
        return n_prev + n_now
    vm_v = after_last(1, (0, 31))                         # barrier in the tail of step 0
    vm_k = after_last(0, (2, K_BARRIER_SLOT - 1))
    assert vm_v < 60 and vm_k < 60
    return vm_v, vm_k


def emit_drain(E, par_last):
    """PV of the final step: V page (parity par_last), keys 96..127, P tile B."""
    for nt in range(2):                                   # row sums of the final step
        E.e(f"v_add_f32 {V(LACC + 2 * nt)}, {V(LACC + 2 * nt)}, {V(TS[nt])}")
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
    E.e(f"s_mov_b32 s{S_LDS0}, %[lds0]")
    E.e(f"s_lshl_b32 s{S_M0B}, %[wave], 10")
    E.e(f"s_add_u32 s{S_M0B}, s{S_M0B}, s{S_LDS0}")
    E.e(f"s_mov_b32 s{S_LASTV}, %[last_valid]")
    for sub in range(4):                                  # clamp(last_valid - 32*sub, 0, 32)
        E.e(f"s_sub_i32 s{S_VLAST + sub}, s{S_LASTV}, {32 * sub}")
        E.e(f"s_max_i32 s{S_VLAST + sub}, s{S_VLAST + sub}, 0")
        E.e(f"s_min_i32 s{S_VLAST + sub}, s{S_VLAST + sub}, 32")
    for sub in range(4):                                  # (-1, 0) where a last page is ragged
        E.e(f"s_cmp_lt_u32 s{S_VLAST + sub}, 32")
        E.e(f"s_cselect_b32 s{S_VLP + 2 * sub}, -1, 0")
        E.e(f"s_mov_b32 s{S_VLP + 2 * sub + 1}, 0")
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
    for nt in range(2):
        E.e(f"v_mov_b32 {V(TS[nt])}, 0")
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
    E.e(f"s_mov_b32 s{S_KKB}, %[kb0]")
    E.e(f"s_mov_b32 s{S_KPG}, %[pg0]")
    # ---- K(0), V(0), K(1) in flight; wait for the first two, publish
    for grp in page_address_lines() + v_address_lines():
        for ln in grp:
            E.e(ln)
    emit_issue_page(E, 0, 0)
    emit_issue_page(E, 1, VRING)
    for grp in page_advance_lines():
        for ln in grp:
            E.e(ln)
    emit_issue_page(E, 0, PAGE)
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
    emit_first_reference(E, S_TILE["A"])
    # first operand fragments of step (R=0, parity 0)
    for f in range(D_AHEAD):
        E.e(ds_read_frag(f, frag_source(0, 0, f)))
    E.e(f"s_waitcnt lgkmcnt({D_AHEAD - 2})")

    # ---- main loop, two pages per trip (ring parity is compile-time)
    loop, exit_even, exit_odd, done = (E.label("LOOP"), E.label("EXIT_EVEN"), E.label("EXIT_ODD"),
                                        E.label("DONE"))
    vmcnt = wait_counts()
    E.e(f"{loop}:")
    for par in range(2):
        for R in range(4):
            emit_step(E, R, par, vmcnt)
        E.e(f"s_cmp_eq_u32 s{S_NLEFT}, 0")
        E.e("s_nop 0")
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
    clob = [f"v{i}" for i in range(128, 256) if not 148 <= i <= 151 and i not in (184, 200)] + [f"a{i}" for i in range(0, 128)] + [f"s{i}" for i in range(36, 96)]
    clob_path = out_path.replace("attn_core_gfx950.inc", "attn_core_clobbers.inc")
    with open(clob_path, "w") as f:
        f.write("// Generated by gen_attn_core.py -- do not edit.\n#define CA_CORE_CLOBBERS \\\n")
        for i in range(0, len(clob), 12):
            chunk = ", ".join(f'"{c}"' for c in clob[i:i + 12])
            f.write("  " + chunk + (", \\\n" if i + 12 < len(clob) else "\n"))
    print(f"{out_path}: {len(text)} lines")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "attn_core_gfx950.inc")
