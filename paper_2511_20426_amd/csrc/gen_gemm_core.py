#!/usr/bin/env python3
"""Emits gemm_core_gfx950.inc: the main loop of the bf16 GEMM  Y[M,N] = X[M,K] . W[N,K]^T  used
for the projections either side of the attention (fp32 accumulation in AGPRs).

Workgroup = 4 waves = a 256 x 256 tile of Y; wave (wm, wn) owns 128 x 128 of it as 4 x 4 MFMA
tiles of 32 x 32 (v_mfma_f32_32x32x16_bf16, A = rows of W, B = rows of X, so that a lane ends up
with 4 consecutive n of one m: pairs pack into bf16 words of a row of Y).  All 256 accumulator
registers of a lane are AGPRs.

K is walked in stages of 64 (four MFMA k-steps of 16).  A stage is 32 KB of W rows and 32 KB of X
rows in LDS: 128-byte rows, so that every load instruction fetches whole 128-byte cache lines (with
64-byte rows each line was fetched twice, and the L2 -> L1 path, 64 B/clk per CU, became the
bound).  The eight 16-byte chunks of row r are stored at position c ^ (r & 7), which makes the
operand reads bank-conflict free.  Two stages fit in LDS (128 KB), which alone would leave the
loads less than one stage of lead (measured: 41.5 cycles per MFMA, the waves wait for data); so
the loads go to registers first -- two sets of 64 VGPRs, filled one and two stages before their
stage's buffer falls free -- and are written to LDS right behind the barrier that frees it.  One
barrier per stage, before its last k-step (this stage's last fragments are in registers by
then), makes the next stage visible and frees this stage's buffer.  Operand fragments are
double-buffered in VGPRs and read one k-step ahead.  Instructions are dealt to the 64 MFMA slots
of a stage by the list scheduler of issue_sched.py.

Register map:
  a[0:255]   accumulators, tile (ti over n, tj over m) at a[16*(4*ti+tj) ..]
  v[0:63]    operand fragments: buffer b, operand (0 = W, 1 = X), sub-tile t at v[32b + 16op + 4t ..]
  v64..v79   LDS read addresses: v[64 + 8*buffer + 4*op + kk] (operand op = 0 W / 1 X, k-step kk)
  v80..v95   lane's byte offset from the stage's global base for W loads 0..7, X loads 0..7
  v100..v103 LDS write address of the lane for (buffer, operand): v[100 + 2*buffer + op]
  v[128:191], v[192:255]  the two staging sets: load (op, i) of a stage at v[set + 32*op + 4*i ..]
  v128,v129  also the temporaries of the epilogue
On exit v[0:127] hold the wave's tile as packed bf16 pairs: tile T = 4*ti+tj, pair p (n = 32 ti +
8 (p/2) + 4 (lane/32) + 2 (p%2), +1; m = 32 tj + lane%32) in v[8T + p].
"""
from __future__ import annotations

import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from issue_sched import Atom, quanta, schedule  # noqa: E402

# Timing experiments only (CA_GEMM_ABL in the environment of the build): 2 no LDS operand reads,
# 4 no global loads, 8 no barriers, 16 no LDS writes.  Results are then meaningless; the shipped library uses 0.
ABL = int(os.environ.get("CA_GEMM_ABL", "0"))
TUNE = dict(kv.split("=") for kv in os.environ.get("CA_GEMM_TUNE", "").split(",") if kv)
CAP = 8.2
STAGE = 65536            # bytes of LDS per stage: W part then X part
PART = 32768
N_BUF = 2
ADDR = 64                # + 8*buffer + 4*op + kk
OFFW, OFFX = 80, 88      # +i
TMP = 128

S_BW, S_BX = 36, 38      # global base of the stage being loaded (64-bit each)
S_TRIPS, S_ISS, S_NST, S_INC = 40, 41, 42, 44
WADDR = 100              # + 2*buffer + op
EARLY = int(TUNE.get("early", 4))   # write/load pairs of a stage that sit behind the barrier; the rest follow in the next stage
SET = [128, 192]


def V(n, w=1):
    return f"v{n}" if w == 1 else f"v[{n}:{n + w - 1}]"


def A(n, w=1):
    return f"a{n}" if w == 1 else f"a[{n}:{n + w - 1}]"


def frag(b, op, t):
    return 32 * b + 16 * op + 4 * t


def mfma(b, ti, tj):
    acc = A(16 * (4 * ti + tj), 16)
    return f"v_mfma_f32_32x32x16_bf16 {acc}, {V(frag(b, 0, ti), 4)}, {V(frag(b, 1, tj), 4)}, {acc}"


def read_frag(b, op, t, buf, kk):
    if ABL & 2:
        return "s_nop 0"
    return f"ds_read_b128 {V(frag(b, op, t), 4)}, {V(ADDR + 8 * buf + 4 * op + kk)} offset:{4096 * t}"


def load_lines(st, op, i):
    """Load (op, i) of a stage into staging set st: 8 rows x 128 bytes, 16 bytes per lane."""
    if ABL & 4:
        return ["s_nop 0"]
    base, off = (S_BW, OFFW) if op == 0 else (S_BX, OFFX)
    return [f"global_load_dwordx4 {V(SET[st] + 32 * op + 4 * i, 4)}, {V(off + i)}, s[{base}:{base + 1}]"]


def write_lines(st, buf, op, i):
    if ABL & 16:
        return ["s_nop 0"]
    return [f"ds_write_b128 {V(WADDR + 2 * buf + op)}, {V(SET[st] + 32 * op + 4 * i, 4)} offset:{1024 * i}"]


def advance_lines():
    """The next stage's global bases: 128 bytes on, or unchanged once the last stage has been
    requested (the surplus loads re-read it and are never used)."""
    return [[f"s_cmp_lt_u32 s{S_ISS}, s{S_NST}", f"s_cselect_b32 s{S_INC}, 128, 0", f"s_addc_u32 s{S_ISS}, s{S_ISS}, 0"],
            [f"s_add_u32 s{S_BW}, s{S_BW}, s{S_INC}", f"s_addc_u32 s{S_BW + 1}, s{S_BW + 1}, 0"],
            [f"s_add_u32 s{S_BX}, s{S_BX}, s{S_INC}", f"s_addc_u32 s{S_BX + 1}, s{S_BX + 1}, 0"]]


LOAD_ORDER = [(op, i) for i in range(8) for op in range(2)]
READ_ORDER = [(0, 0), (1, 0), (1, 1), (1, 2), (1, 3), (0, 1), (0, 2), (0, 3)]   # as the MFMAs need them


def build_stage(P):
    """Stage P (mod 2) of the steady state: 64 slots of (MFMA, lines issued after it)."""
    buf = P % N_BUF
    mf, tail = [], [[] for _ in range(64)]
    for kk in range(4):
        for ti in range(4):
            for tj in range(4):
                mf.append(mfma(kk & 1, ti, tj))
    for i in (15, 31, 63):
        tail[i] += ["s_waitcnt lgkmcnt(0)"]
    # before the last k-step: this stage's last fragments are in registers, last stage's LDS writes
    # are done (lgkmcnt), and stage P+2 has arrived in its staging set (the 16 loads behind it may fly)
    tail[47] += ["s_waitcnt vmcnt(16) lgkmcnt(0)"] + ([] if ABL & 8 else ["s_barrier"])
    atoms = []
    for kk in range(4):
        nbuf, nkk = (buf, kk + 1) if kk < 3 else (1 - buf, 0)
        prev = None
        for k, (op, t) in enumerate(READ_ORDER):
            prev = Atom([read_frag((kk + 1) & 1, op, t, nbuf, nkk)], 16 * kk, 16 * kk + k,
                        [prev] if prev else [], 0, hard=16 * kk + 12)
            atoms.append(prev)
    # A staging register quad is written to LDS and refilled at once: pair k = (write k of the
    # stage two ahead of the buffer's, load k of the stage two further on).  Pairs 0..EARLY-1 sit
    # behind the barrier (this stage's buffer, set P % 2), the others in the next stage's slots
    # 0..44 -- here: the other buffer's.  A load leads its write by exactly two stages.
    for k, (op, i) in enumerate(LOAD_ORDER[EARLY:]):
        at = 1 + (k * 43) // (16 - EARLY)
        atoms.append(Atom(write_lines(1 - buf, 1 - buf, op, i) + load_lines(1 - buf, op, i), at, at, hard=44))
    prev = None
    for grp in advance_lines():
        prev = Atom(grp, 48, 48, [prev] if prev else [], 0, hard=50)
        atoms.append(prev)
    for k, (op, i) in enumerate(LOAD_ORDER[:EARLY]):
        at = 49 + (k * 14) // EARLY
        atoms.append(Atom(write_lines(buf, buf, op, i) + load_lines(buf, op, i), at, at, [prev], 0, hard=62))
    fixed = [2.0 + sum(quanta(l) for l in tail[i]) for i in range(64)]
    placed = schedule(fixed, atoms, CAP)
    out = []
    for i in range(64):
        lines = []
        for a in placed[i]:
            lines += a.lines
        out.append((mf[i], lines + tail[i]))
    # LDS operations complete in order: a k-step's fragments have landed once no more LDS
    # operations are outstanding than were issued behind the last of its reads
    for end in (15, 31, 63):
        behind = 0
        done = False
        for i in range(end, end - 16, -1):
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
    # every VGPR input is copied out first: the inputs may live in v[96:127], which holds WADDR
    names = [f"offw{i}" for i in range(8)] + [f"offx{i}" for i in range(8)] + ["aw0", "ax0", "waddr"]
    tmp = {n: SET[0] + k for k, n in enumerate(names)}
    for n in names:
        e(f"v_mov_b32 {V(tmp[n])}, %[{n}]")
    for i in range(8):
        e(f"v_mov_b32 {V(OFFW + i)}, {V(tmp[f'offw{i}'])}")
        e(f"v_mov_b32 {V(OFFX + i)}, {V(tmp[f'offx{i}'])}")
    for buf in range(N_BUF):
        for op, name in ((0, "aw0"), (1, "ax0")):
            for kk in range(4):                           # chunk index of k-step kk = that of 0, xor 2 kk
                r = ADDR + 8 * buf + 4 * op + kk
                e(f"v_xor_b32 {V(r)}, {kk << 5}, {V(tmp[name])}")
                e(f"v_add_u32 {V(r)}, %[lds0], {V(r)}")
                e(f"v_add_u32 {V(r)}, {buf * STAGE + op * PART}, {V(r)}")
    for buf in range(N_BUF):
        for op in range(2):
            e(f"v_add_u32 {V(WADDR + 2 * buf + op)}, {buf * STAGE + op * PART}, {V(tmp['waddr'])}")
    for r in range(256):
        e(f"v_accvgpr_write_b32 {A(r)}, 0")
    # stages 0 and 1 into the staging sets; stage 0 and the first pairs of stage 1 on into LDS
    # (the loop's first stage writes the rest); stage 2 into set 0, first pairs of stage 3 into set 1
    for st in range(2):
        if st:
            for grp in advance_lines():
                L.extend(grp)
        for op, i in LOAD_ORDER:
            L.extend(load_lines(st, op, i))
    e("s_waitcnt vmcnt(0)")
    for op, i in LOAD_ORDER:
        L.extend(write_lines(0, 0, op, i))
    for op, i in LOAD_ORDER[:EARLY]:
        L.extend(write_lines(1, 1, op, i))
    for grp in advance_lines():
        L.extend(grp)
    for op, i in LOAD_ORDER:
        L.extend(load_lines(0, op, i))
    for grp in advance_lines():
        L.extend(grp)
    for op, i in LOAD_ORDER[:EARLY]:
        L.extend(load_lines(1, op, i))
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
    e("s_nop 15\ns_nop 15\ns_nop 15")                      # the last MFMAs have written back
    for T in range(16):
        for p in range(8):
            e(f"v_accvgpr_read_b32 {V(TMP)}, {A(16 * T + 2 * p)}")
            e(f"v_accvgpr_read_b32 {V(TMP + 1)}, {A(16 * T + 2 * p + 1)}")
            e(f"v_cvt_pk_bf16_f32 {V(8 * T + p)}, {V(TMP)}, {V(TMP + 1)}")
    return L


def main(out_path):
    text = []
    for ln in generate():
        text.extend(ln.split("\n"))
    with open(out_path, "w") as f:
        f.write("// Generated by gen_gemm_core.py -- do not edit.\n")
        for t in text:
            f.write('"' + t + '\\n"\n')
    clob = [f"v{i}" for i in range(128, 256)] + [f"a{i}" for i in range(256)] + [f"s{i}" for i in range(36, 48)]
    with open(out_path.replace("gemm_core_gfx950.inc", "gemm_core_clobbers.inc"), "w") as f:
        f.write("// Generated by gen_gemm_core.py -- do not edit.\n#define CA_GEMM_CLOBBERS \\\n")
        for i in range(0, len(clob), 12):
            chunk = ", ".join(f'"{c}"' for c in clob[i:i + 12])
            f.write("  " + chunk + (", \\\n" if i + 12 < len(clob) else "\n"))
    print(f"{out_path}: {len(text)} lines")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "gemm_core_gfx950.inc")
