#!/usr/bin/env python3
"""Writes mainloop_asm.h: the inline-assembly text of the MFMA kernel's K loop (gfx950).

Run `python gen_mainloop.py > mainloop_asm.h` after changing the schedule; the generated
header is committed, the build does not run this script.

The loop is a ping-pong between the two wave groups of a workgroup (waves 0-3 and 4-7; the
hardware places wave w and wave w+4 on the same SIMD).  Per K step of 64 a group alternates
between a memory phase (32 LDS fragment reads for the whole step) and an MFMA phase (32
v_mfma_f32_32x32x16_bf16 with no waits); the groups are offset by one phase, with an s_barrier
between phases, so each SIMD's matrix pipe always has one wave issuing MFMAs while the other
wave fetches.  Global->LDS tile loads (global_load_lds_dwordx4, 8 per wave per K step) go
into the stage both groups have finished reading: group 0 issues them in its memory phase,
group 1 between the MFMAs of its MFMA phase.

Register plan per wave: v[0:127] accumulators acc[mi][ni] = v[16*(2*mi+ni) ..+15];
v[128:191] A fragments fa[kk][mi] = v[128+4*(4*kk+mi) ..+3]; v[192:223] B fragments
fb[kk][ni] = v[192+4*(2*kk+ni) ..+3]; v[224:227] A read addresses per kk.
SGPRs: s[40:41] / s[42:43] pointers to the next A / B tile to load, s44 this wave's LDS write
base in the stage being filled, s45 K steps left, s46 pointer advances left (the pointer stops
at the last full tile: loads issued past it re-read that tile into a stage nobody reads any
more), s47 B pointer step in bytes, s48-s50 temporaries.
"""
import sys

STAGE_A = 0x8000      # bytes of the A tile inside a stage; a stage is 0x10000 bytes


def acc(mi, ni):
    b = 16 * (2 * mi + ni)
    return f"v[{b}:{b + 15}]"


def fa(kk, mi):
    b = 128 + 4 * (4 * kk + mi)
    return f"v[{b}:{b + 3}]"


def fb(kk, ni, half=None):
    b = 192 + 4 * (2 * kk + ni)
    if half is None:
        return f"v[{b}:{b + 3}]"
    return f"v[{b + 2 * half}:{b + 2 * half + 1}]"


def setup():
    # the A read address of k-substep kk differs from that of substep 0 by kk*32 XORed in
    return ["v_mov_b32 v224, %[ard]",
            "v_xor_b32 v225, 32, %[ard]",
            "v_xor_b32 v226, 64, %[ard]",
            "v_xor_b32 v227, 0x60, %[ard]"]


def ds_reads():
    out = []
    for kk in range(4):
        for mi in range(4):
            out.append(f"ds_read_b128 {fa(kk, mi)}, v{224 + kk} offset:{mi * 4096}")
        for ni in range(2):
            for rd in range(2):
                out.append(f"ds_read_b64_tr_b16 {fb(kk, ni, rd)}, %[brd{ni}] offset:{kk * 8192 + rd * 2048}")
    return out


def toggles():
    """Point the fragment reads at the other stage."""
    out = [f"v_xor_b32 v{224 + kk}, 0x10000, v{224 + kk}" for kk in range(4)]
    out += ["v_xor_b32 %[brd0], 0x10000, %[brd0]", "v_xor_b32 %[brd1], 0x10000, %[brd1]"]
    return out


def load(j):
    """Wave-instruction j of a tile: 1 KiB, 16 bytes per lane, straight into LDS at m0 + lane*16."""
    if j < 4:
        return [f"s_add_u32 m0, s44, {j * 1024}", "s_nop 0", f"global_load_lds_dwordx4 %[ao{j}], s[40:41]"]
    return [f"s_add_u32 m0, s44, {STAGE_A + (j - 4) * 1024}", "s_nop 0",
            f"global_load_lds_dwordx4 %[bo{j - 4}], s[42:43]"]


def advance():
    return ["s_cmp_lg_u32 s46, 0",
            "s_cselect_b32 s48, 128, 0",
            "s_cselect_b32 s49, s47, 0",
            "s_cselect_b32 s50, 1, 0",
            "s_add_u32 s40, s40, s48", "s_addc_u32 s41, s41, 0",
            "s_add_u32 s42, s42, s49", "s_addc_u32 s43, s43, 0",
            "s_sub_u32 s46, s46, s50",
            "s_xor_b32 s44, s44, 0x10000"]


def mfmas(loads_after=None):
    out, i = [], 0
    for kk in range(4):
        for mi in range(4):
            for ni in range(2):
                # rhs fragment as first operand: the accumulator gets 4 consecutive n per lane
                out.append(f"v_mfma_f32_32x32x16_bf16 {acc(mi, ni)}, {fb(kk, ni)}, {fa(kk, mi)}, {acc(mi, ni)}")
                if loads_after and i in loads_after:
                    out += load(loads_after[i])
                i += 1
    return out


def group0():
    s = setup() + ["L0_top_%=:"] + ds_reads()
    for j in range(8):
        s += load(j)
    s += advance() + toggles()
    s += ["s_waitcnt lgkmcnt(0)", "s_barrier"]
    s += mfmas()
    s += ["s_waitcnt vmcnt(0)", "s_barrier",
          "s_sub_u32 s45, s45, 1", "s_cmp_lg_u32 s45, 0", "s_cbranch_scc1 L0_top_%=",
          "s_nop 15", "s_nop 15"]
    return s


def group1():
    s = setup() + ["s_barrier", "L1_top_%=:"] + ds_reads() + toggles()
    s += ["s_waitcnt vmcnt(0) lgkmcnt(0)", "s_barrier"]
    s += mfmas({1 + 4 * j: j for j in range(8)})
    s += advance()
    s += ["s_sub_u32 s45, s45, 1", "s_cmp_lg_u32 s45, 0", "s_cbranch_scc0 L1_end_%=",
          "s_barrier", "s_branch L1_top_%=", "L1_end_%=:", "s_nop 15", "s_nop 15"]
    return s


def macro(name, lines):
    return f"#define {name} \\\n" + " \\\n".join('  "' + l + '\\n\\t"' for l in lines)


def main():
    clob = ", ".join(f'"v{i}"' for i in range(128, 228))
    out = ["// Generated by gen_mainloop.py -- do not edit by hand.", "#pragma once",
           macro("GSPMD_MAINLOOP_G0", group0()), macro("GSPMD_MAINLOOP_G1", group1()),
           f'#define GSPMD_MAINLOOP_CLOBBERS {clob}, "s48", "s49", "s50", "m0", "scc", "vcc", "memory"']
    sys.stdout.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
