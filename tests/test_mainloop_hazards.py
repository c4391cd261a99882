"""CPU model of the memory ordering of the generated K loop (csrc/gen_mainloop.py).

Every wave's instruction stream is executed in the scalar interpreter of test_mainloop_schedule, extended to follow
which LDS stage each read address register points at.  Barriers cut the streams into epochs that all eight waves of a
workgroup pass together.  Checked over whole workgroups (four waves of group 0 with four of group 1, every loop
variant):
  * read after write: a tile part is read only in an epoch after the one in which every wave that loads a piece of
    it has waited for those loads (vmcnt counts loads in issue order);
  * write after read: a load into a stage is issued only in an epoch after the last read of the tile that the stage
    held before;
  * a wave reaches a barrier with no LDS read outstanding (the fragments are in registers before the MFMAs start, and
    the reads of a stage are over before the barrier that frees it);
  * every read goes to the stage of the tile it is meant to read;
  * a wave leaves the loop with no tile load in flight and with its last LDS read before the last barrier both groups
    pass (the kernel's epilogue reuses LDS without a further barrier).
The model cannot see timing, only what the waits and barriers guarantee."""
import re

import pytest

from tests.test_mainloop_schedule import MASK, NSTAGE, STAGE, STAGE_A, generator, initial


def trace(lines, sgpr, outstanding):
    """Events of one wave: ('load', epoch, stage, part, serial), ('done', epoch, serial), ('read', epoch, stage, part, src, step).
    `outstanding`: serials of loads in flight when the loop starts (oldest first)."""
    labels = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    s, scc, m0, pc, epoch = dict(sgpr), 0, None, 0, 0
    vreg, ev, queue, serial, lds_pending, nk = {}, [], list(outstanding), 1000, 0, sgpr["s45"]

    def val(x):
        x = x.strip()
        if x == "m0":
            return m0
        return s[x] if x.startswith("s") else int(x, 0)

    n = 0
    while pc < len(lines):
        n += 1
        assert n < 500000
        l = lines[pc]
        pc += 1
        if l.endswith(":"):
            continue
        op, _, rest = l.partition(" ")
        a = [t.strip() for t in rest.split(",")] if rest else []
        if op == "v_add_u32":                       # read address = stage offset + per-lane offset inside the stage
            assert a[2] in ("%[ard]", "%[brd]")
            vreg[a[0]] = (a[2], s[a[1]], a[1])
        elif op == "v_xor_b32":                     # a constant below the part size: same stage, same part
            assert int(a[1], 0) < STAGE_A
            vreg[a[0]] = vreg[a[2]]
        elif op.startswith("ds_read"):
            addr = a[1].split()[0]
            name, stage_off, src = vreg[addr]
            assert stage_off % STAGE == 0 and int(re.search(r"offset:(\d+)", l).group(1)) < STAGE_A
            ev.append(("read", epoch, stage_off // STAGE, "A" if name == "%[ard]" else "B", src, nk - s["s45"]))
            lds_pending += 1
        elif op.startswith("v_mfma") or op == "s_nop":
            continue
        elif op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", rest)
            if m:
                while len(queue) > int(m.group(1)):
                    ev.append(("done", epoch, queue.pop(0)))
            if "lgkmcnt(0)" in rest:
                lds_pending = 0
        elif op == "s_barrier":
            assert lds_pending == 0, "a wave reaches a barrier with LDS reads outstanding"
            epoch += 1
        elif op == "global_load_lds_dwordx4":
            rel = m0 - s["s44"]
            ev.append(("load", epoch, rel // STAGE, "A" if rel % STAGE < STAGE_A else "B", serial))
            queue.append(serial)
            serial += 1
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
            raise AssertionError("instruction the model does not know: " + l)
    return ev, queue, epoch


@pytest.mark.parametrize("layout", range(4))
@pytest.mark.parametrize("nbm0,nbm", [(8, 8), (8, 7), (8, 6), (8, 5), (8, 4), (6, 4), (4, 4)])
@pytest.mark.parametrize("nk64", [1, 2, 3, 4, 7, 12])
def test_waits_and_barriers_order_every_tile_load_and_read(layout, nbm0, nbm, nk64):
    g = generator()
    # per tile part: epoch from which it may be read, epochs in which it is read, epoch in which it is overwritten
    readable, reads, written = {}, {}, {}
    for t in range(4):                       # the kernel's prologue loads tiles 0-3; tiles 0 and 1 have landed and the
        for part in "AB":                    # prologue's barrier has published them when the loop starts
            readable[(t, part)] = 0 if t < 2 else None
    epochs = set()
    for grp in (0, 1):
        for w in range(4):
            sg = initial(grp, w, nk64)[0]
            lines = g.group0(w, layout, nbm0) if grp == 0 else g.group1(w, layout, nbm)
            # in flight at loop start: this wave's 8 pieces of tile 2 (group 0) or 3 (group 1), serials 0-7
            ev, left, last_epoch = trace(lines, sg, range(8))
            epochs.add(last_epoch)
            assert not left, "a tile load is still in flight when the wave leaves the loop"
            # the wave's last LDS read lies before the last barrier it shares with the other group (group 1 passes no
            # barrier after its last MFMA phase), so LDS may be reused right after the loop without another barrier
            assert max(e[1] for e in ev if e[0] == "read") < 2 * nk64
            batch_of = {}                     # load serial -> tile
            nload = 0
            for e in ev:
                if e[0] == "load":
                    tile = 4 + grp + 2 * (nload // 8)
                    nload += 1
                    batch_of[e[4]] = (tile, e[3])
                    assert e[2] == tile % NSTAGE
                    written.setdefault((tile, e[3]), []).append(e[1])
                elif e[0] == "done":
                    key = (2 + grp, None) if e[2] < 8 else batch_of[e[2]]
                    for part in ("AB" if key[1] is None else key[1]):
                        k = (key[0], part)
                        readable[k] = max(readable.get(k) or 0, e[1] + 1)
                elif e[0] == "read":
                    _, epoch, stage, part, src, step = e
                    # a K-major part is addressed through the per-tile stage ring, a K-contiguous one through the ring of
                    # the half that holds the wave's rows
                    assert src == ({"A": "s53" if layout & 1 else "s55", "B": "s56" if layout & 2 else "s53"}[part])
                    if src == "s53":          # K-major part: the tile's own stage, tiles 2u and 2u+1 in turn
                        tile = 2 * step + (0 if stage == (2 * step) % NSTAGE else 1)
                    elif src == "s55":        # K-contiguous lhs: the half that holds this group's rows
                        tile = 2 * step + grp
                    else:                     # K-contiguous rhs: the half that holds this wave's columns
                        assert src == "s56"
                        tile = 2 * step + (w >> 1)
                    assert stage == tile % NSTAGE, (grp, w, step, src)
                    reads.setdefault((tile, part), []).append(epoch)
    assert len(epochs) == 1                  # every wave passes the same number of barriers
    nkt = 2 * nk64
    for (tile, part), eps in reads.items():
        assert tile < nkt
        assert readable.get((tile, part)) is not None, ("read of a tile whose loads were never waited for", tile, part)
        assert min(eps) >= readable[(tile, part)], ("read before the loads were waited for and published", tile, part)
    for (tile, part), eps in written.items():
        before = reads.get((tile - NSTAGE, part))
        if before:
            assert min(eps) > max(before), ("a stage is overwritten while its tile may still be read", tile, part)
    # every tile of the loop is read from both parts
    assert {t for t, _ in reads} == set(range(nkt))
