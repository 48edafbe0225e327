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
the operand reads (16 rows x one chunk per quarter wave) bank-conflict free.  Two stages fit in
LDS (128 KB), which alone would leave the loads less than one stage of lead; so the loads go to a
staging set of 64 VGPRs first, one stage before their buffer falls free, and each register quad is
written to LDS and refilled at once (a load leads its write by exactly one stage).  One barrier
per stage, before its last k-step (this stage's last fragments are in registers by then), makes
the next stage visible and frees this stage's buffer.  Operand fragments are double-buffered in
VGPRs and read one k-step ahead.  Instructions are dealt to the 128 MFMA slots of a stage by the
list scheduler of issue_sched.py.

Register map:
  a[0:255]   accumulators, tile (ti over n, tj over m) at a[4*(8*ti+tj) ..]
  v[0:127]   operand fragments: buffer b, operand (0 = W, 1 = X), sub-tile t at v[64b + 32op + 4t ..]
  v[128:191] the staging set: load (op, i) of a stage at v[128 + 32*op + 4*i ..]
  v192..v199 LDS read addresses: v[192 + 4*buffer + 2*op + kk] (operand op = 0 W / 1 X, k-step kk)
  v200..v215 lane's byte offset from the stage's global base for W loads 0..7, X loads 0..7
  v216..v219 LDS write address of the lane for (buffer, operand): v[216 + 2*buffer + op]
  v220..v222 temporaries of the set-up and the epilogue
On exit v[0:127] hold the wave's tile as packed bf16 pairs: tile T = 8*ti+tj, pair p (n = 16 ti +
4 (lane/16) + 2 p, +1; m = 16 tj + lane%16) in v[2T + p].
"""
from __future__ import annotations

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from issue_sched import Atom, quanta, schedule  # noqa: E402

# Timing experiments only (CA_GEMM_ABL in the environment of the build): 2 no LDS operand reads,
# 4 no global loads, 8 no barriers, 16 no LDS writes.  Results are then meaningless; the shipped
# library uses 0.
ABL = int(os.environ.get("CA_GEMM_ABL", "0"))
TUNE = dict(kv.split("=") for kv in os.environ.get("CA_GEMM_TUNE", "").split(",") if kv)
CAP = float(TUNE.get("cap", 4.2))   # issue quanta between two MFMAs of 16 cycles
STAGE = 65536            # bytes of LDS per stage: W part then X part
PART = 32768
N_BUF = 2
SLOTS = 128              # MFMAs per stage and wave: 2 k-steps x 8 x 8 tiles

SET = 128
ADDR = 192               # + 4*buffer + 2*op + kk
OFFW, OFFX = 200, 208    # +i
WADDR = 216              # + 2*buffer + op
TMP = 220

S_BW, S_BX = 36, 38      # global base of the stage being loaded (64-bit each)
S_TRIPS, S_ISS, S_NST, S_INC = 40, 41, 42, 44


def V(n, w=1):
    return f"v{n}" if w == 1 else f"v[{n}:{n + w - 1}]"


def A(n, w=1):
    return f"a{n}" if w == 1 else f"a[{n}:{n + w - 1}]"


def frag(b, op, t):
    return 64 * b + 32 * op + 4 * t


def mfma(b, ti, tj):
    acc = A(4 * (8 * ti + tj), 4)
    return f"v_mfma_f32_16x16x32_bf16 {acc}, {V(frag(b, 0, ti), 4)}, {V(frag(b, 1, tj), 4)}, {acc}"


def read_frag(b, op, t, buf, kk):
    if ABL & 2:
        return "s_nop 0"
    return f"ds_read_b128 {V(frag(b, op, t), 4)}, {V(ADDR + 4 * buf + 2 * op + kk)} offset:{2048 * t}"


def load_lines(op, i):
    """Load (op, i) of a stage into the staging set: 8 rows x 128 bytes, 16 bytes per lane."""
    if ABL & 4:
        return ["s_nop 0"]
    base, off = (S_BW, OFFW) if op == 0 else (S_BX, OFFX)
    return [f"global_load_dwordx4 {V(SET + 32 * op + 4 * i, 4)}, {V(off + i)}, s[{base}:{base + 1}]"]


def write_lines(buf, op, i):
    """The quad's previous contents, loaded one stage ago, go to LDS: at most the 15 younger
    loads may still be in flight."""
    if ABL & 16:
        return ["s_nop 0"]
    return ["s_waitcnt vmcnt(15)",
            f"ds_write_b128 {V(WADDR + 2 * buf + op)}, {V(SET + 32 * op + 4 * i, 4)} offset:{1024 * i}"]


def advance_lines():
    """The next stage's global bases: 128 bytes on, or unchanged once the last stage has been
    requested (the surplus loads re-read it and are never used)."""
    return [[f"s_cmp_lt_u32 s{S_ISS}, s{S_NST}", f"s_cselect_b32 s{S_INC}, 128, 0", f"s_addc_u32 s{S_ISS}, s{S_ISS}, 0"],
            [f"s_add_u32 s{S_BW}, s{S_BW}, s{S_INC}", f"s_addc_u32 s{S_BW + 1}, s{S_BW + 1}, 0"],
            [f"s_add_u32 s{S_BX}, s{S_BX}, s{S_INC}", f"s_addc_u32 s{S_BX + 1}, s{S_BX + 1}, 0"]]


LOAD_ORDER = [(op, i) for i in range(8) for op in range(2)]
# fragments in the order the MFMAs (ti outer, tj inner) first need them
READ_ORDER = [(0, 0)] + [(1, t) for t in range(8)] + [(0, t) for t in range(1, 8)]
HALF = 8                 # write/load pairs behind the barrier; the other 8 in the next stage's first k-step


def pair_atoms(buf, op, i, at, after, hard):
    """wait, write the quad to LDS, refill it: three atoms in consecutive slots from `at`."""
    lines = write_lines(buf, op, i)
    out, prev = [], None
    for k, grp in enumerate([lines[:1], lines[1:], load_lines(op, i)]):
        if not grp:
            continue
        prev = Atom(grp, at + k, at + k, ([prev] if prev else list(after)), 0, hard=hard + k)
        out.append(prev)
    return out


def build_stage(P):
    """Stage P (mod 2) of the steady state: SLOTS slots of (MFMA, lines issued after it)."""
    buf = P % N_BUF
    half = SLOTS // 2
    mf, tail = [], [[] for _ in range(SLOTS)]
    for kk in range(2):
        for ti in range(8):
            for tj in range(8):
                mf.append(mfma(kk, ti, tj))
    # before the last k-step: this stage's last fragments are in registers and the writes of the
    # next stage's data are done (lgkmcnt 0); after the barrier this stage's buffer is free
    tail[half - 1] += ["s_waitcnt lgkmcnt(0)"] + ([] if ABL & 8 else ["s_barrier"])
    tail[SLOTS - 1] += ["s_waitcnt lgkmcnt(0)"]
    atoms = []
    for kk in range(2):
        nbuf, nkk = (buf, 1) if kk == 0 else (1 - buf, 0)
        prev = None
        for k, (op, t) in enumerate(READ_ORDER):
            at = half * kk + 1 + 3 * k
            prev = Atom([read_frag(1 - kk, op, t, nbuf, nkk)], at, at, [prev] if prev else [], 0,
                        hard=half * kk + half - 6)
            atoms.append(prev)
    # A staging quad is written to LDS and refilled at once.  Pairs HALF..15 finish the stage that
    # becomes visible at this stage's barrier (other buffer); pairs 0..HALF-1, behind the barrier,
    # start the stage after it (this stage's buffer), and the bases move on first.
    for k, (op, i) in enumerate(LOAD_ORDER[HALF:]):
        at = 2 + 6 * k
        atoms += pair_atoms(1 - buf, op, i, at, [], half - 6)
    prev = None
    for grp in advance_lines():
        prev = Atom(grp, half, half, [prev] if prev else [], 0, hard=half + 4)
        atoms.append(prev)
    for k, (op, i) in enumerate(LOAD_ORDER[:HALF]):
        at = half + 5 + 6 * k
        atoms += pair_atoms(buf, op, i, at, [prev], SLOTS - 6)
    fixed = [2.0 + sum(quanta(l) for l in tail[i]) for i in range(SLOTS)]
    placed = schedule(fixed, atoms, CAP)
    out = []
    for i in range(SLOTS):
        lines = []
        for a in placed[i]:
            lines += a.lines
        out.append((mf[i], lines + tail[i]))
    # LDS operations complete in order: a k-step's fragments have landed once no more LDS
    # operations are outstanding than were issued behind the last of its reads
    end = SLOTS - 1
    behind, done = 0, False
    for i in range(end, half - 1, -1):
        for ln in reversed(out[i][1]):
            if ln.startswith("ds_read"):
                done = True
                break
            if ln.startswith("ds_write"):
                behind += 1
        if done:
            break
    m, lines = out[end]
    out[end] = (m, [f"s_waitcnt lgkmcnt({behind})" if ln == "s_waitcnt lgkmcnt(0)" else ln for ln in lines])
    return out


def generate():
    L = []
    e = L.append
    e(f"s_mov_b64 s[{S_BW}:{S_BW + 1}], %[base_w]")
    e(f"s_mov_b64 s[{S_BX}:{S_BX + 1}], %[base_x]")
    e(f"s_mov_b32 s{S_NST}, %[n_stages]")
    e(f"s_lshr_b32 s{S_TRIPS}, s{S_NST}, 1")
    e(f"s_mov_b32 s{S_ISS}, 1")
    # every VGPR input is copied out first: the inputs may live anywhere in v[0:127]
    names = [f"offw{i}" for i in range(8)] + [f"offx{i}" for i in range(8)] + ["aw0", "ax0", "waddr"]
    dst = {f"offw{i}": OFFW + i for i in range(8)}
    dst.update({f"offx{i}": OFFX + i for i in range(8)})
    dst.update({"aw0": TMP, "ax0": TMP + 1, "waddr": TMP + 2})
    for n in names:
        e(f"v_mov_b32 {V(dst[n])}, %[{n}]")
    for buf in range(N_BUF):
        for op, name in ((0, "aw0"), (1, "ax0")):
            for kk in range(2):                           # chunk index of k-step 1 = that of 0, xor 4
                r = ADDR + 4 * buf + 2 * op + kk
                e(f"v_xor_b32 {V(r)}, {kk << 6}, {V(dst[name])}")
                e(f"v_add_u32 {V(r)}, %[lds0], {V(r)}")
                e(f"v_add_u32 {V(r)}, {buf * STAGE + op * PART}, {V(r)}")
    for buf in range(N_BUF):
        for op in range(2):
            e(f"v_add_u32 {V(WADDR + 2 * buf + op)}, {buf * STAGE + op * PART}, {V(dst['waddr'])}")
    for r in range(256):
        e(f"v_accvgpr_write_b32 {A(r)}, 0")
    # Stage 0 through the staging set into buffer 0; stage 1 into the set, its first HALF quads on
    # into buffer 1 and refilled with stage 2 (the loop's first stage does the rest).
    for op, i in LOAD_ORDER:
        L.extend(load_lines(op, i))
    e("s_waitcnt vmcnt(0)")
    for op, i in LOAD_ORDER:
        L.extend(write_lines(0, op, i))
    for grp in advance_lines():
        L.extend(grp)
    for op, i in LOAD_ORDER:
        L.extend(load_lines(op, i))
    e("s_waitcnt vmcnt(0)")
    for grp in advance_lines():
        L.extend(grp)
    for op, i in LOAD_ORDER[:HALF]:
        L.extend(write_lines(1, op, i))
        L.extend(load_lines(op, i))
    e("s_waitcnt lgkmcnt(0)")
    e("s_barrier")
    for op, t in READ_ORDER:
        e(read_frag(0, op, t, 0, 0))
    e("s_waitcnt lgkmcnt(0)")
    e("LOOP_%=:")
    for P in range(N_BUF):
        e(f"; ---- stage {P}")
        for m, lines in build_stage(P):
            e(m)
            L.extend(lines)
    e(f"s_sub_u32 s{S_TRIPS}, s{S_TRIPS}, 1")
    e(f"s_cmp_lg_u32 s{S_TRIPS}, 0")
    e("s_nop 0")
    e("s_cbranch_scc1 LOOP_%=")
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
