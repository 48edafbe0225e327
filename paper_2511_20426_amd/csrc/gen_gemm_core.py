#!/usr/bin/env python3
"""Emits gemm_core_gfx950.inc: the main loop of the bf16 GEMM  Y[M,N] = X[M,K] . W[N,K]^T  used
for the projections either side of the attention (fp32 accumulation in AGPRs).

Workgroup = 4 waves = a 256 x 256 tile of Y; wave (wm, wn) owns 128 x 128 of it as 8 x 8 MFMA
tiles of 16 x 16 (v_mfma_f32_16x16x32_bf16, A = rows of W, B = rows of X, so that a lane ends up
with 4 consecutive n of one m: pairs pack into bf16 words of a row of Y).  All 256 accumulator
registers of a lane are AGPRs.  The 16x16x32 shape is chosen for power: the chip is power-limited
under a full MFMA load, and per flop this shape reads and writes half as many accumulator
registers as 32x32x16 (an MFMA-only loop with toggling operands sustains 2.4 PFLOP/s at 2.38 GHz
with it, 2.1 at 2.05 GHz with 32x32x16); its price is issue room -- an MFMA of 16 cycles leaves two
issue quanta of 4 cycles free instead of six per 32 -- which this loop can afford.

K is walked in stages of 64 (two MFMA k-steps of 32).  A stage is 32 KB of W rows and 32 KB of X
rows in LDS: 128-byte rows, so that every load instruction fetches whole 128-byte cache lines (with
64-byte rows each line was fetched twice, and the L2 -> L1 path, 64 B/clk per CU, became the
bound).  The eight 16-byte chunks of row r are stored at position c ^ ((r >> 1) & 7), which makes
the operand reads (16 rows x one chunk per quarter wave) bank-conflict free.  Both operands stream
global -> LDS with global_load_lds_dwordx4 (no registers, and far cheaper for the LDS pipe than
ds_write: with register staging the waves waited for LDS).  All 160 KB of LDS are used: a ring of
three stages for W and of two for X.  One barrier per stage, before its last k-step (this stage's
last fragments are in registers by then), makes the next stage visible and frees this stage's
buffers; right behind it go the loads of X for stage s+2 (into the buffer just freed, one stage of
lead) and of W for stage s+3 (two stages of lead).  Loads complete in order, so "everything but the
eight W loads issued last" (vmcnt 8) is what the barrier waits for.  Operand fragments are
double-buffered in VGPRs and read one k-step ahead.  Instructions are dealt to the 128 MFMA slots
of a stage by the list scheduler of issue_sched.py.

Register map:
  a[0:255]   accumulators, tile (ti over n, tj over m) at a[4*(8*ti+tj) ..]
  v[0:127]   operand fragments: buffer b, operand (0 = W, 1 = X), sub-tile t at v[64b + 32op + 4t ..]
  v192..v197 LDS read addresses of W: v[192 + 2*ring slot + kk];  v198..v201 of X: v[198 + 2*ring slot + kk]
  v202..v209, v210..v217  lane's byte offset from the stage's global base for W / X loads 0..7
  v220..v222 temporaries of the set-up and the epilogue
On exit v[0:127] hold the wave's tile as packed bf16 pairs: tile T = 8*ti+tj, pair p (n = 16 ti +
4 (lane/16) + 2 p, +1; m = 16 tj + lane%16) in v[2T + p].
"""
from __future__ import annotations

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from issue_sched import Atom, quanta, schedule  # noqa: E402

CAP = 4.2                # issue quanta between two MFMAs of 16 cycles
PART = 32768             # bytes of one operand's rows of one stage
NW, NX = 3, 2            # ring depths; LDS = [W ring][X ring] = 160 KB
XBASE = NW * PART
PERIOD = 6               # stages after which both rings are back where they were
SLOTS = 128              # MFMAs per stage and wave: 2 k-steps x 8 x 8 tiles

ADDRW, ADDRX = 192, 198  # + 2*ring slot + kk
OFFW, OFFX = 202, 210    # +i
TMP = 220

S_BW, S_BX = 36, 38      # global bases of the W / X stage being loaded (64-bit each)
S_TRIPS, S_ISS, S_NST, S_M0B, S_INC, S_XISS = 40, 41, 42, 43, 44, 45


def V(n, w=1):
    return f"v{n}" if w == 1 else f"v[{n}:{n + w - 1}]"


def A(n, w=1):
    return f"a{n}" if w == 1 else f"a[{n}:{n + w - 1}]"


def frag(b, op, t):
    return 64 * b + 32 * op + 4 * t


def mfma(b, ti, tj):
    acc = A(4 * (8 * ti + tj), 4)
    return f"v_mfma_f32_16x16x32_bf16 {acc}, {V(frag(b, 0, ti), 4)}, {V(frag(b, 1, tj), 4)}, {acc}"


def read_frag(b, op, t, stage, kk):
    addr = (ADDRW + 2 * (stage % NW) if op == 0 else ADDRX + 2 * (stage % NX)) + kk
    return f"ds_read_b128 {V(frag(b, op, t), 4)}, {V(addr)} offset:{2048 * t}"


def load_lines(op, stage, i):
    """Load i (0..7) of this wave's share of a stage of W (op 0) or X (op 1): 8 rows x 128 bytes
    -> 1 KB of LDS."""
    ring = (stage % NW) * PART if op == 0 else XBASE + (stage % NX) * PART
    base, off = (S_BW, OFFW) if op == 0 else (S_BX, OFFX)
    return [f"s_add_u32 m0, s{S_M0B}, {ring + 1024 * i}",
            f"global_load_lds_dwordx4 {V(off + i)}, s[{base}:{base + 1}]"]


def advance_lines(base, counter):
    """The next stage's global base: 128 bytes on, or unchanged once the last stage has been
    requested (the surplus loads re-read it and are never used)."""
    return [[f"s_cmp_lt_u32 s{counter}, s{S_NST}", f"s_cselect_b32 s{S_INC}, 128, 0", f"s_addc_u32 s{counter}, s{counter}, 0"],
            [f"s_add_u32 s{base}, s{base}, s{S_INC}", f"s_addc_u32 s{base + 1}, s{base + 1}, 0"]]


# fragments in the order the MFMAs (ti outer, tj inner) first need them
READ_ORDER = [(0, 0)] + [(1, t) for t in range(8)] + [(0, t) for t in range(1, 8)]
X_BY = 40               # the 8 X loads of a stage issue within this many slots behind the barrier


def build_stage(P):
    """Stage P (mod PERIOD) of the steady state: SLOTS slots of (MFMA, lines issued after it)."""
    half = SLOTS // 2
    mf, tail = [], [[] for _ in range(SLOTS)]
    for kk in range(2):
        for ti in range(8):
            for tj in range(8):
                mf.append(mfma(kk, ti, tj))
    # before the last k-step: this stage's last fragments are in registers; everything but the
    # W loads issued last has landed; behind the barrier this stage's buffers are free
    tail[half - 1] += ["s_waitcnt vmcnt(@VM@) lgkmcnt(0)", "s_barrier"]
    tail[SLOTS - 1] += ["s_waitcnt lgkmcnt(0)"]
    atoms = []
    for kk in range(2):
        nstage, nkk = (P, 1) if kk == 0 else (P + 1, 0)
        prev = None
        for k, (op, t) in enumerate(READ_ORDER):
            at = half * kk + 1 + 3 * k
            prev = Atom([read_frag(1 - kk, op, t, nstage, nkk)], at, at, [prev] if prev else [], 0,
                        hard=half * kk + half - 6)
            atoms.append(prev)
    # behind the barrier: X of stage P+2 first (it is needed one stage on), then W of stage P+3
    prev = None
    for grp in advance_lines(S_BX, S_XISS) + advance_lines(S_BW, S_ISS):
        prev = Atom(grp, half, half, [prev] if prev else [], 0, hard=half + 6)
        atoms.append(prev)
    last = prev
    for i in range(8):
        at = half + 4 + (i * X_BY) // 8
        last = Atom(load_lines(1, P + 2, i), at, at, [last], 0, hard=half + X_BY + 6)
        atoms.append(last)
    for i in range(8):
        at = half + 6 + 7 * i
        last = Atom(load_lines(0, P + 3, i), at, at, [last] if i == 0 else [prev], 0, hard=SLOTS - 3)
        atoms.append(last)
    fixed = [2.0 + sum(quanta(l) for l in tail[i]) for i in range(SLOTS)]
    placed = schedule(fixed, atoms, CAP)
    out = []
    for i in range(SLOTS):
        lines = []
        for a in placed[i]:
            lines += a.lines
        out.append((mf[i], lines + tail[i]))
    # Loads complete in order.  At the next barrier the X loads issued here must have landed (and
    # with them every older load): as many loads may still fly as were issued behind the last X load.
    kinds = ["x" if f"s[{S_BX}:" in ln else "w" for _, lines in out for ln in lines if ln.startswith("global_load_lds")]
    behind = len(kinds) - 1 - max(k for k, x in enumerate(kinds) if x == "x") if "x" in kinds else 0
    out = [(m, [ln.replace("@VM@", str(behind)) for ln in lines]) for m, lines in out]
    return out


def generate():
    L = []
    e = L.append
    e(f"s_mov_b64 s[{S_BW}:{S_BW + 1}], %[base_w]")
    e(f"s_mov_b64 s[{S_BX}:{S_BX + 1}], %[base_x]")
    e(f"s_mov_b32 s{S_NST}, %[n_stages]")
    e(f"s_lshr_b32 s{S_TRIPS}, s{S_NST}, 1")
    e(f"s_mov_b32 s{S_ISS}, 1")
    e(f"s_mov_b32 s{S_XISS}, 1")
    e(f"s_lshl_b32 s{S_M0B}, %[wave], 13")
    e(f"s_add_u32 s{S_M0B}, s{S_M0B}, %[lds0]")
    dst = {f"offw{i}": OFFW + i for i in range(8)}
    dst.update({f"offx{i}": OFFX + i for i in range(8)})
    dst.update({"aw0": TMP, "ax0": TMP + 1})
    for n, r in dst.items():
        e(f"v_mov_b32 {V(r)}, %[{n}]")
    for name, areg, depth, ring0 in (("aw0", ADDRW, NW, 0), ("ax0", ADDRX, NX, XBASE)):
        for slot in range(depth):
            for kk in range(2):                           # chunk index of k-step 1 = that of 0, xor 4
                r = areg + 2 * slot + kk
                e(f"v_xor_b32 {V(r)}, {kk << 6}, {V(dst[name])}")
                e(f"v_add_u32 {V(r)}, %[lds0], {V(r)}")
                e(f"v_add_u32 {V(r)}, {ring0 + slot * PART}, {V(r)}")
    for r in range(256):
        e(f"v_accvgpr_write_b32 {A(r)}, 0")
    # W stages 0, 1, 2 and X stages 0, 1 on their way; everything lands; first fragments
    for st in range(NW):
        if st:
            for grp in advance_lines(S_BW, S_ISS):
                L.extend(grp)
        for i in range(8):
            L.extend(load_lines(0, st, i))
    for st in range(NX):
        if st:
            for grp in advance_lines(S_BX, S_XISS):
                L.extend(grp)
        for i in range(8):
            L.extend(load_lines(1, st, i))
    e("s_waitcnt vmcnt(0)")
    e("s_barrier")
    for op, t in READ_ORDER:
        e(read_frag(0, op, t, 0, 0))
    e("s_waitcnt lgkmcnt(0)")
    # the trip count is checked every two stages; a loop trip is PERIOD stages
    e("LOOP_%=:")
    for P in range(PERIOD):
        e(f"; ---- stage {P}")
        for m, lines in build_stage(P):
            e(m)
            L.extend(lines)
        if P % 2 == 1:
            e(f"s_sub_u32 s{S_TRIPS}, s{S_TRIPS}, 1")
            e(f"s_cmp_lg_u32 s{S_TRIPS}, 0")
            e("s_nop 0")
            e("s_cbranch_scc1 LOOP_%=" if P == PERIOD - 1 else "s_cbranch_scc0 DONE_%=")
    e("DONE_%=:")
    e("s_waitcnt vmcnt(0)")                                # surplus loads have landed
    e("s_nop 15")
    e("s_nop 15")                                          # the last MFMAs have written back
    for T in range(64):
        for p in range(2):
            e(f"v_accvgpr_read_b32 {V(TMP)}, {A(4 * T + 2 * p)}")
            e(f"v_accvgpr_read_b32 {V(TMP + 1)}, {A(4 * T + 2 * p + 1)}")
            e(f"v_cvt_pk_bf16_f32 {V(2 * T + p)}, {V(TMP)}, {V(TMP + 1)}")
    return L


def main(out_path):
    text = []
    for ln in generate():
        text.extend(ln.split("\n"))
    with open(out_path, "w") as f:
        f.write("// Generated by gen_gemm_core.py -- do not edit.\n")
        for t in text:
            f.write('"' + t + '\\n"\n')
    clob = [f"v{i}" for i in range(128, 224)] + [f"a{i}" for i in range(256)] + [f"s{i}" for i in range(36, 48)]
    with open(out_path.replace("gemm_core_gfx950.inc", "gemm_core_clobbers.inc"), "w") as f:
        f.write("// Generated by gen_gemm_core.py -- do not edit.\n#define CA_GEMM_CLOBBERS \\\n")
        for i in range(0, len(clob), 12):
            chunk = ", ".join(f'"{c}"' for c in clob[i:i + 12])
            f.write("  " + chunk + (", \\\n" if i + 12 < len(clob) else "\n"))
    print(f"{out_path}: {len(text)} lines")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "gemm_core_gfx950.inc")
