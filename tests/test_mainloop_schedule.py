"""CPU checks of the generated assembly main loop (csrc/gen_mainloop.py -> csrc/mainloop_asm.h).

The loop's scalar bookkeeping (tile pointers, LDS stage ring, loop counter) is executed in a small SALU interpreter
and compared with closed forms: which tile every load instruction fetches, where in LDS it lands, that no load is
issued for a tile past the loop's last one (the bug class that reads out of bounds), and that the two wave groups execute
the same number of barriers (the bug class that hangs).  Also: the committed header is what the generator writes."""
import importlib.util
import os
import re
import subprocess
import sys

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2105_04663_amd", "csrc")
MASK = 0xFFFFFFFF
STAGE, STAGE_A, NSTAGE = 0x8000, 0x4000, 5


def generator():
    spec = importlib.util.spec_from_file_location("gen_mainloop", os.path.join(CSRC, "gen_mainloop.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def run(lines, sgpr):
    """Interpret the scalar instructions of one macro; returns the events (loads, barriers, waits) and final SGPRs."""
    labels = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    s, scc, m0, ev, pc, steps = dict(sgpr), 0, None, [], 0, 0

    def val(x):
        x = x.strip()
        if x == "m0":
            return m0
        return s[x] if x.startswith("s") else int(x, 0)

    while pc < len(lines):
        steps += 1
        assert steps < 500000, "the loop does not terminate"
        l = lines[pc]
        pc += 1
        if l.endswith(":"):
            continue
        op, _, rest = l.partition(" ")
        a = [t.strip() for t in rest.split(",")] if rest else []
        if op.startswith("v_") or op.startswith("ds_read") or op == "s_nop":
            continue
        if op == "s_waitcnt":
            ev.append(("wait", rest))
        elif op == "s_barrier":
            ev.append(("barrier",))
        elif op == "global_load_lds_dwordx4":
            lo = int(re.match(r"s\[(\d+):", a[1]).group(1))
            ev.append(("load", m0, s[f"s{lo}"] | (s[f"s{lo + 1}"] << 32), a[0]))
        elif op in ("s_add_u32", "s_addc_u32", "s_sub_u32"):
            x, y = val(a[1]), val(a[2])
            if op == "s_sub_u32":
                r, c = x - y, int(y > x)
            else:
                r = x + y + (scc if op == "s_addc_u32" else 0)
                c = r >> 32
            r &= MASK
            if a[0] == "m0":
                m0 = r
            else:
                s[a[0]] = r
            scc = int(bool(c))
        elif op == "s_cmp_lg_u32":
            scc = int(val(a[0]) != val(a[1]))
        elif op == "s_cmp_ge_u32":
            scc = int(val(a[0]) >= val(a[1]))
        elif op == "s_cmp_gt_u32":
            scc = int(val(a[0]) > val(a[1]))
        elif op == "s_cmp_le_u32":
            scc = int(val(a[0]) <= val(a[1]))
        elif op == "s_cselect_b32":
            s[a[0]] = val(a[1]) if scc else val(a[2])
        elif op == "s_cbranch_scc1":
            pc = labels[a[0]] if scc else pc
        elif op == "s_cbranch_scc0":
            pc = labels[a[0]] if not scc else pc
        elif op == "s_branch":
            pc = labels[a[0]]
        else:
            raise AssertionError("instruction the interpreter does not know: " + l)
    return ev, s


A0, B0, ASTEP, BSTEP = 0x7F_F0000000, 0x11_FFFFF000, 128, 0x123400     # B crosses a 4 GiB boundary: carries matter


def initial(grp, w, nk64):
    nkt = 2 * nk64
    first = min(4 + grp, nkt - 1)
    a, b = A0 + (first >> 1) * ASTEP, B0 + first * (BSTEP // 2)
    sg = {f"s{i}": 0 for i in range(40, 60)}
    sg.update(s40=a & MASK, s41=a >> 32, s42=b & MASK, s43=b >> 32, s44=0x400 + w * 4096, s45=nk64,
              s46=(nkt - 1 - first) // 2, s47=BSTEP, s54=ASTEP, s52=((4 + grp) % NSTAGE) * STAGE, s53=0,
              s55=grp * STAGE, s56=(w >> 1) * STAGE)
    return sg, a, b


@pytest.mark.parametrize("layout", range(4))
@pytest.mark.parametrize("grp,nbm", [(0, 8), (0, 6), (0, 4), (1, 8), (1, 7), (1, 6), (1, 5), (1, 4)])
def test_tile_loads_land_where_the_kernel_reads_them_and_stay_in_bounds(layout, grp, nbm):
    g = generator()
    for w in range(4):
        for nk64 in (1, 2, 3, 4, 5, 9, 16):
            sg, a0, b0 = initial(grp, w, nk64)
            lines = g.group0(w, layout, nbm) if grp == 0 else g.group1(w, layout, nbm)
            assert sum(l.startswith("v_mfma") for l in lines) == 2 * 8 * nbm     # the step with loads and its copy without
            ev, end = run(lines, sg)
            loads = [e for e in ev if e[0] == "load"]
            nload = max(nk64 - 2, 0)                          # the last two steps have no tile left to load
            assert len(loads) == 8 * nload                    # one tile (8 instructions of this wave) per loading step
            nadv = sg["s46"]
            assert nadv == max(nload - 1, 0)                  # so the pointers never move past the last tile loaded
            for u in range(nload):
                step_loads = loads[8 * u:8 * u + 8]
                adv = min(u, nadv)
                stage = ((4 + grp + 2 * u) % NSTAGE) * STAGE
                want = set()
                for j in range(4):
                    want.add((sg["s44"] + stage + j * 1024, a0 + adv * ASTEP, f"%[ao{j}]"))
                    want.add((sg["s44"] + stage + STAGE_A + j * 1024, b0 + adv * BSTEP, f"%[bo{j}]"))
                assert {(m0, base, opnd) for _, m0, base, opnd in step_loads} == want, (w, nk64, u)
            assert end["s45"] == 0


@pytest.mark.parametrize("layout", range(4))
def test_both_wave_groups_execute_the_same_number_of_barriers(layout):
    g = generator()
    for w in range(4):
        for nk64 in (1, 2, 3, 8):
            for nbm0 in (4, 6, 8):
                n0 = sum(e[0] == "barrier" for e in run(g.group0(w, layout, nbm0), initial(0, w, nk64)[0])[0])
                for nbm in (4, 5, 6, 7, 8):
                    n1 = sum(e[0] == "barrier" for e in run(g.group1(w, layout, nbm), initial(1, w, nk64)[0])[0])
                    assert n0 == n1 == 2 * nk64


def test_read_stage_ring_visits_the_tiles_in_order():
    # s53 (K-major parts) advances one stage per tile, s55/s56 (K-contiguous halves) two per step, all modulo 5 stages
    g = generator()
    for layout in range(4):
        _, end = run(g.group0(0, layout), initial(0, 0, 7)[0])
        assert end["s53"] == (14 % NSTAGE) * STAGE
        if not layout & 1:
            assert end["s55"] == (14 % NSTAGE) * STAGE
        if layout & 2:
            assert end["s56"] == (14 % NSTAGE) * STAGE


def test_committed_header_is_the_generators_output():
    out = subprocess.run([sys.executable, os.path.join(CSRC, "gen_mainloop.py")], capture_output=True, text=True, check=True).stdout
    assert out == open(os.path.join(CSRC, "mainloop_asm.h")).read()
