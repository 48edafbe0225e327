"""CPU tests of the code generators of the hand-scheduled kernels: the list scheduler honours its
constraints, and the emitted instruction streams keep the invariants the kernels rely on (hazard
distances, condition-code lifetimes, load / barrier / wait bookkeeping).  Nothing is assembled or
run here; the GPU parity tests cover what the code computes."""
import importlib.util
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_20426_amd", "csrc")


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


sched = _load("issue_sched")
attn = _load("gen_attn_core")
gemm = _load("gen_gemm_core")

SCC_WRITERS = ("s_add", "s_sub", "s_cmp", "s_and", "s_or", "s_mul", "s_lsh", "s_min", "s_max")


def test_scheduler_respects_ready_order_gaps_and_hard_deadlines():
    rng = np.random.default_rng(7)
    for trial in range(20):
        n = 32
        atoms = []
        for k in range(40):
            after = [atoms[j] for j in rng.choice(len(atoms), size=min(len(atoms), int(rng.integers(0, 3))), replace=False)] if atoms else []
            ready = int(rng.integers(0, 20))
            atoms.append(sched.Atom(["v_add_f32 v0, v0, v0"] * int(rng.integers(1, 3)), ready, int(rng.integers(ready, n)),
                                    after, int(rng.integers(0, 3)), hard=n - 1))
        placed = sched.schedule([2.0] * n, atoms, 8.0)
        assert sorted(id(a) for s in placed for a in s) == sorted(id(a) for a in atoms)     # each exactly once
        pos = {id(a): (i, k) for i, s in enumerate(placed) for k, a in enumerate(s)}
        for a in atoms:
            assert a.slot == pos[id(a)][0] and a.slot >= a.ready
            for dep, gap in a.after:
                assert a.slot >= dep.slot + gap
                assert pos[id(a)] > pos[id(dep)]                                             # issue order too
        for i, s in enumerate(placed):                                                         # no overflow: all of it fits
            assert 2.0 + sum(a.cost for a in s) <= 8.0 + 1e-9 or any(a.hard <= i for a in s)
    # an atom larger than any slot takes the first one that holds nothing else; one that finds no
    # room before its hard deadline is placed there regardless
    big = sched.Atom(["v_exp_f32 v1, v2"] * 5, 2, 3, hard=5)
    small = [sched.Atom(["v_add_f32 v0, v0, v0"] * 6, 0, 0, hard=7) for _ in range(3)]
    placed = sched.schedule([2.0] * 8, small + [big], 8.0)
    assert big.slot == 3 and [a.slot for a in small] == [0, 1, 2] and placed[3] == [big]
    late = sched.Atom(["v_add_f32 v0, v0, v0"] * 4, 0, 0, hard=1)
    placed = sched.schedule([2.0] * 4, [sched.Atom(["v_add_f32 v0, v0, v0"] * 6, 0, 0, hard=3) for _ in range(2)] + [late], 8.0)
    assert late.slot == 1


def test_quanta_model():
    q = sched.quanta
    assert q("v_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]") == 2.0
    assert q("v_exp_f32 v1, v2") == 2.0 and q("ds_read_b128 v[0:3], v4 offset:16") == 2.2
    assert q("global_load_lds_dwordx4 v1, s[2:3]") == 2.7 and q("s_cbranch_scc1 X") == 2.5
    assert q("s_waitcnt lgkmcnt(0)") == 1.0 and q("LABEL_1:") == 0.0 and q("; comment") == 0.0


def _steps():
    return [(R, par, attn.build_step(R, par)) for par in range(2) for R in range(4)]


def test_attention_step_invariants():
    exp_re = re.compile(r"v_exp_f32 (v\d+), (v\d+)")
    for R, par, (slots, cold) in _steps():
        assert len(slots) == 32 and all(m.startswith("v_mfma_f32_32x32x16_bf16") for m, _ in slots)
        flat = [(i, ln) for i, (m, lines) in enumerate(slots) for ln in [m] + lines]
        text = [ln for _, ln in flat]
        # 32 exponentials, 16 packs, row-sum adds for every probability exactly once
        exps = {m.group(1): i for i, ln in flat for m in [exp_re.match(ln)] if m}
        assert len(exps) == 32
        packs = [(i, ln) for i, ln in flat if ln.startswith("v_cvt_pk_bf16_f32")]
        assert len(packs) == 16
        used = []
        for i, ln in flat:
            if ln.startswith(("v_cvt_pk_bf16_f32", "v_add_f32")):
                for reg in re.findall(r"v\d+", ln.split(",", 1)[1]):
                    if reg in exps:
                        assert i >= exps[reg] + 2, (R, ln)      # a trans result is consumed >= 2 slots later
                        used.append((ln.split()[0], reg))
        assert sorted(r for op, r in used if op == "v_cvt_pk_bf16_f32") == sorted(exps)
        assert sorted(r for op, r in used if op == "v_add_f32") == sorted(exps)
        # scc set by the s_or survives until the branch that ends the step
        k_or = max(k for k, ln in enumerate(text) if ln.startswith("s_or_b64"))
        k_br = max(k for k, ln in enumerate(text) if ln.startswith("s_cbranch_scc1"))
        assert k_br > k_or + 1                                  # not directly behind the s_or
        assert not any(ln.split()[0].startswith(SCC_WRITERS) for ln in text[k_or + 1:k_br])
        # the compare that feeds it sits at least a slot before
        i_cmp = max(i for i, ln in flat if ln.startswith("v_cmp_lt_f32 vcc"))
        i_or = max(i for i, ln in flat if ln.startswith("s_or_b64"))
        assert i_or >= i_cmp + 1
        # scc producer / consumer pairs are adjacent (no other scc writer between)
        for k, ln in enumerate(text):
            if ln.split()[0] in ("s_cselect_b32", "s_cselect_b64", "s_addc_u32"):
                back = k - 1
                while text[back].split()[0] in ("s_cselect_b32", "s_cselect_b64"):
                    back -= 1
                assert text[back].split()[0].startswith(("s_cmp", "s_add_u32", "s_addc_u32")), (R, text[back], ln)
        # every M0 write is directly followed by its load
        for k, ln in enumerate(text):
            if ln.startswith("s_add_u32 m0"):
                assert text[k + 1].startswith("global_load_lds_dwordx4")


def test_attention_page_traffic_bookkeeping():
    """16 loads per page pair (8 V after the V barrier, 8 K after the K barrier), two barriers per
    page, and the vmcnt operands equal the number of loads issued behind the page being awaited."""
    vm_v, vm_k = attn.wait_counts()
    events = []                                   # ("load", stream) | ("bar", which), in program order over one page
    for R in range(4):
        slots, _ = attn.build_step(R, 0)
        for m, lines in slots:
            for k, ln in enumerate(lines):
                if ln.startswith("global_load_lds"):
                    events.append(("load", "V" if "s[76:77]" in ln else "K"))
                if ln == "s_barrier":
                    wait = lines[k - 1]
                    events.append(("bar", "V" if "@VMCNT_V@" in wait else "K"))
    loads = [e[1] for e in events if e[0] == "load"]
    assert loads.count("V") == 8 and loads.count("K") == 8
    assert [e[1] for e in events if e[0] == "bar"] == ["V", "K"]           # V barrier ends step 0, K barrier in step 2
    two = events + events                         # two consecutive pages
    for which, vm in (("V", vm_v), ("K", vm_k)):
        bars = [k for k, e in enumerate(two) if e == ("bar", which)]
        b = bars[1]                               # a barrier in the second page: awaits the loads of the first
        first_page_last = max(k for k, e in enumerate(events) if e == ("load", which))
        # every load of that stream in the previous period has at most vm loads behind it
        behind = sum(1 for e in two[first_page_last + 1:b] if e[0] == "load")
        # loads of the awaited page issued after the previous barrier of the same kind are the ones meant
        assert behind == vm, (which, behind, vm)


def test_attention_cold_blocks_have_no_barrier_and_return():
    lines = attn.generate()
    text = [p for ln in lines for p in ln.split("\n")]
    n_bar = sum(1 for ln in text if ln == "s_barrier")
    assert n_bar == 1 + 2 * 2                     # prologue + two per page, two pages per loop trip
    colds = [k for k, ln in enumerate(text) if ln.startswith("COLD_")]
    assert len(colds) == 8
    for k in colds:
        j = k
        while not text[j].startswith("s_branch BACK_"):
            assert text[j] != "s_barrier"
            j += 1


def test_gemm_stage_invariants():
    for P in range(gemm.PERIOD):
        slots = gemm.build_stage(P)
        assert len(slots) == 128 and all(m.startswith("v_mfma_f32_16x16x32_bf16") for m, _ in slots)
        text = [ln for m, lines in slots for ln in [m] + lines]
        reads = [ln for ln in text if ln.startswith("ds_read_b128")]
        loads = [k for k, ln in enumerate(text) if ln.startswith("global_load_lds_dwordx4")]
        assert len(reads) == 32 and len(loads) == 16
        assert sum(1 for ln in text if ln == "s_barrier") == 1
        k_bar = text.index("s_barrier")
        # all loads sit behind the barrier that frees their buffers; every M0 write is directly
        # followed by its load; W goes to ring slot (P+3) % 3, X to ring slot (P+2) % 2
        assert min(loads) > k_bar
        for k in loads:
            m0 = re.match(r"s_add_u32 m0, s\d+, (\d+)$", text[k - 1])
            assert m0, text[k - 1]
            off = int(m0.group(1))
            if f"s[{gemm.S_BX}:" in text[k]:
                assert gemm.XBASE + ((P + 2) % gemm.NX) * gemm.PART <= off < gemm.XBASE + ((P + 2) % gemm.NX + 1) * gemm.PART
            else:
                assert ((P + 3) % gemm.NW) * gemm.PART <= off < ((P + 3) % gemm.NW + 1) * gemm.PART
        # the wait at the barrier lets exactly the loads issued behind the last X load fly
        kinds = ["x" if f"s[{gemm.S_BX}:" in text[k] else "w" for k in loads]
        behind = len(kinds) - 1 - max(i for i, x in enumerate(kinds) if x == "x")
        assert text[k_bar - 1] == f"s_waitcnt vmcnt({behind}) lgkmcnt(0)"
        assert kinds.count("x") == 8 and kinds.count("w") == 8
        # fragment reads: first k-step reads this stage's ring slots, second the next stage's
        for ln in text[:k_bar]:
            if ln.startswith("ds_read_b128"):
                addr = int(re.search(r", v(\d+) offset", ln).group(1))
                assert addr in (gemm.ADDRW + 2 * (P % gemm.NW) + 1, gemm.ADDRX + 2 * (P % gemm.NX) + 1)
        for ln in text[k_bar:]:
            if ln.startswith("ds_read_b128"):
                addr = int(re.search(r", v(\d+) offset", ln).group(1))
                assert addr in (gemm.ADDRW + 2 * ((P + 1) % gemm.NW), gemm.ADDRX + 2 * ((P + 1) % gemm.NX))
        assert text[-1] == "s_waitcnt lgkmcnt(0)"
        # the two k-steps use different fragment buffers; every accumulator tile is hit once per k-step
        for kk in range(2):
            accs = [re.match(r"v_mfma\S+ (a\[\d+:\d+\])", m_).group(1) for m_, _ in slots[64 * kk:64 * kk + 64]]
            assert len(set(accs)) == 64
