#!/usr/bin/env python3
"""Writes mainloop_asm.h: the inline-assembly text of the MFMA kernel's K loop (gfx950).

Run `python gen_mainloop.py > mainloop_asm.h` after changing the schedule; the generated header is committed,
the build does not run this script.

Shape of the loop.  K advances in steps of 64 = two LDS tiles of 32.  LDS has five 32 KiB stages (tile t lives in
stage t % 5: A part and B part of 16 KiB each, formats below).  The workgroup's two wave groups (waves 0-3 and 4-7; wave
w and w+4 share a SIMD) alternate, one phase apart and separated by s_barrier, between
  * a read phase: all fragments of one K step, 32 LDS reads (16 ds_read_b128 for A, 16 ds_read_b64_tr_b16 for B)
    into 96 VGPRs, and
  * an MFMA phase: 64 v_mfma_f32_16x16x32_bf16 with no waits,
so that each SIMD's matrix pipe always has exactly one wave issuing MFMAs (two waves issuing at once share the pipe
badly: measured 64 % pipe efficiency with one wave starved).  Inside an MFMA phase the 4 column blocks of each row block
are visited back and forth, so that consecutive MFMAs share one fragment operand (the chip is power-limited and operand
switching costs: +1.4 % on the feed-forward share and +1.1 % on the experts' over restarting every row block at
column block 0, same box; column blocks outermost with the row blocks back and forth gains 1.0 %).  16x16x32 is used rather than 32x32x16 because it moves
half the accumulator registers per flop and the chip is power-limited: a pure MFMA loop on N(0,1) data sustains
1996 TFLOP/s with 16x16x32 and 1700 with 32x32x16 (both reach 2480 on all-zero data).
Global->LDS tile loads (global_load_lds_dwordx4, 1 KiB per wave-instruction) are issued only from MFMA phases, one
after every 6th MFMA and staggered by wave, so the CU's texture-address unit (about one such load per 16 cycles) sees
an even stream and never stalls an MFMA wave; a whole tile is loaded by the four waves of ONE group: group 0 loads
tile 2u+4 during the MFMA phase of step u, group 1 tile 2u+5.  With five stages every load has at least one full
phase (>= 1024 cycles) plus the slack of a read phase to land.  The last two K steps have no tile left to load: they run
a second copy of the step without loads (and without the pointer bookkeeping), so that nothing is fetched twice and the
loop ends with no load in flight.
The end of an MFMA phase is the loop's critical path (the other group's MFMAs wait at the barrier for it), so
nothing but the barrier follows the last MFMA: the loads are all issued by MFMA 46, and the scalar bookkeeping of the
phase (pointer advance, stage ring, loop counter, s_waitcnt vmcnt for the tile this barrier publishes) is spread, one
instruction after each MFMA, over MFMAs 48-62; the LDS write base of the next phase is formed before the barrier that
starts it.  This was worth 4 % over doing the bookkeeping after the last MFMA.  The bookkeeping passes values through SCC
(compare -> select, add -> add with carry), so only MFMAs may be interleaved with it, never a tile load (whose
s_add_u32 of M0 overwrites SCC); tests/test_mainloop_schedule.py executes the scalar stream of every macro in an
interpreter and checks pointers, LDS destinations and barrier counts against closed forms.
Arriving at the barrier a few MFMAs early instead (so that the other group's first MFMAs overlap this group's last)
is slower by 4-6 %: two waves issuing MFMAs on one SIMD at once is what the alternation exists to avoid.

Operand layouts.  Each operand's LDS tile keeps the operand's own memory order, so there are two tile formats.
K-major (rows of 256 m resp. n): the part of tile t is [32 k][256 columns]; a fragment is two ds_read_b64_tr_b16,
block b of 16 columns at address ^ (b << 5).
K-contiguous: the two parts of K step u (tiles 2u and 2u+1) hold the operand's 256 rows as two halves of
[128 rows][64 k] -- rows 0-127 in tile 2u's part, rows 128-255 in tile 2u+1's -- so that a row is a whole 128-byte
line of global memory (a [256][32] part would fetch half lines and cost the texture-address unit twice the lookups per
load instruction).  A wave reads all its K-contiguous fragments of the step from ONE part (the half its rows are in;
stage offset in s55 for the lhs, s56 for the rhs, advancing two stages per step): one ds_read_b128 per fragment, the
second 32 k at address ^ 64.  Who loads what, and when a stage is free again, is the same as for K-major parts: the
part of tile t is loaded with tile t, by group t & 1, and stage t % 5 is last read in the read phase of group 1.
The forward einsums have a K-contiguous lhs and a K-major rhs; a weight gradient has both K-major, an input gradient
both K-contiguous.  One set of macros is written per combination (GSPMD_MAINLOOP_L<layout>_..., layout bit 0 = lhs
K-major, bit 1 = rhs K-contiguous); only the read phase differs (32, 48, 24 or 40 LDS reads into the same 96 fragment
registers).
Partly valid tiles: when the rows an output tile owns end inside group 1's half (rows 128-255), its waves run a
variant (..._G1R4_... to ..._G1R7_...) that reads and multiplies only the first 4 to 7 of their 8 row blocks; the rest of
their accumulators stays zero and is never stored.  When they end inside group 0's half (a problem with at most 128
rows), group 0 runs ..._G0R4_... or ..._G0R6_... and group 1 its shortest variant (it still loads its share of every
tile and passes every barrier).  The loads are the same in every variant; only their spacing between the MFMAs
shrinks with the phase.

Register plan per wave: v[0:127] accumulators acc(bm, bn) = v[4*(4*bm+bn) ..+3] (bm = 16-row block 0..7 of the
wave's 128 rows, bn = 16-column block 0..3 of its 64 columns); fragments of tile q (0/1) of the K step:
A fa_q[bm] = v[128+48q+4bm ..+3], B fb_q[bn] = v[160+48q+4bn ..+3]; v224 A read address, v225..v228 B read
addresses (per bn) in the stage being read, v229/v230 A read addresses of blocks 1..7 of a K-major lhs (an LDS read
takes its address when it issues, so the two registers alternate).
SGPRs: s[40:41]/s[42:43] pointers to the next A/B tile this group loads, s44 this wave's LDS write base (stage 0),
s45 K steps left, s46 pointer advances left (the pointers stop at the last tile that is loaded), s47/s54 B/A pointer step in bytes (two tiles), s52 write-stage offset,
s53 read-stage offset (K-major parts), s55/s56 read-stage offsets of a K-contiguous lhs/rhs, s48-s51 temporaries.
"""
import sys

STAGE = 0x8000
STAGE_A = 0x4000
NSTAGE = 5
LDS = STAGE * NSTAGE


def acc(bm, bn):
    b = 4 * (4 * bm + bn)
    return f"v[{b}:{b + 3}]"


def fa(q, bm, half=None):
    b = 128 + 48 * q + 4 * bm
    if half is None:
        return f"v[{b}:{b + 3}]"
    return f"v[{b + 2 * half}:{b + 2 * half + 1}]"


def fb(q, bn, half=None):
    b = 160 + 48 * q + 4 * bn
    if half is None:
        return f"v[{b}:{b + 3}]"
    return f"v[{b + 2 * half}:{b + 2 * half + 1}]"


def xor_const(dst, c, src):
    return f"v_xor_b32 {dst}, {c if c <= 64 else hex(c)}, {src}"


def read_addrs(layout, q):
    """Address registers for the reads of tile q (0/1) of the step."""
    out = []
    if layout & 1:          # K-major lhs: stage of tile 2u+q
        out.append("v_add_u32 v224, s53, %[ard]")
    elif q == 0:            # K-contiguous lhs: this wave's half, both tiles' k from one part
        out += ["v_add_u32 v224, s55, %[ard]", xor_const("v229", 64, "v224")]
    if not layout & 2:      # K-major rhs: one address per 16-column block
        out.append("v_add_u32 v225, s53, %[brd]")
        out += [xor_const(f"v{225 + bn}", bn << 5, "v225") for bn in range(1, 4)]
    elif q == 0:
        out += ["v_add_u32 v225, s56, %[brd]", xor_const("v226", 64, "v225")]
    return out


def ds_reads(q, layout, nbm=8):
    out = []
    for bm in range(nbm):
        if layout & 1:      # K-major lhs: block bm at address ^ (bm << 5), formed in one of two alternating registers
            reg = "v224" if bm == 0 else f"v{229 + (bm & 1)}"
            if bm:
                out.append(xor_const(reg, bm << 5, "v224"))
            for rd in range(2):
                out.append(f"ds_read_b64_tr_b16 {fa(q, bm, rd)}, {reg} offset:{rd * 2048}")
        else:
            out.append(f"ds_read_b128 {fa(q, bm)}, {'v229' if q else 'v224'} offset:{bm * 2048}")
    for bn in range(4):
        if layout & 2:
            out.append(f"ds_read_b128 {fb(q, bn)}, {'v226' if q else 'v225'} offset:{bn * 2048}")
        else:
            for rd in range(2):
                out.append(f"ds_read_b64_tr_b16 {fb(q, bn, rd)}, v{225 + bn} offset:{rd * 2048}")
    return out


def step_stage(reg, n):
    return [f"s_add_u32 {reg}, {reg}, {STAGE * n}", f"s_sub_u32 s48, {reg}, {LDS}", f"s_cmp_ge_u32 {reg}, {LDS}", f"s_cselect_b32 {reg}, s48, {reg}"]


def mem_phase(layout, nbm=8):
    out = (read_addrs(layout, 0) + ds_reads(0, layout, nbm) + step_stage("s53", 1)
           + read_addrs(layout, 1) + ds_reads(1, layout, nbm) + step_stage("s53", 1))
    if not layout & 1:
        out += step_stage("s55", 2)
    if layout & 2:
        out += step_stage("s56", 2)
    return out


def load(j):
    if j < 4:
        return [f"s_add_u32 m0, s49, {j * 1024}", "s_nop 0", f"global_load_lds_dwordx4 %[ao{j}], s[40:41]"]
    return [f"s_add_u32 m0, s49, {STAGE_A + (j - 4) * 1024}", "s_nop 0", f"global_load_lds_dwordx4 %[bo{j - 4}], s[42:43]"]


def advance():
    """Next tile of this group (two tiles on), pointers frozen at the last full tile; next write stage."""
    return ["s_cmp_lg_u32 s46, 0",
            "s_cselect_b32 s50, s54, 0",
            "s_cselect_b32 s51, s47, 0",
            "s_cselect_b32 s48, 1, 0",
            "s_sub_u32 s46, s46, s48",
            "s_add_u32 s40, s40, s50", "s_addc_u32 s41, s41, 0",
            "s_add_u32 s42, s42, s51", "s_addc_u32 s43, s43, 0"] + step_stage("s52", 2)


LOAD_STRIDE = {8: 6, 7: 5, 6: 4, 5: 3, 4: 2}      # MFMAs between two tile loads of a wave, by row blocks computed


def mfma_phase(w, tail, nbm=8, loads=True):
    """8 * nbm MFMAs (all 8 row blocks of the wave, or only the first nbm when the rest of its rows lies beyond the valid
    extent).  With `loads`, tile loads go after MFMAs stride * j + (wave-dependent offset), all issued 16 MFMAs before
    the end, and the pointer / stage bookkeeping follows; `tail` (loop counter, wait) comes last.  All of that is spread,
    one scalar instruction after each MFMA, over the last 16 MFMAs, so that nothing but the barrier comes after the
    last one.  Only MFMAs are interleaved with the bookkeeping: it passes values through SCC (compare -> select,
    add -> add-with-carry), which the s_add_u32 of a tile load would overwrite."""
    n = 8 * nbm
    st = LOAD_STRIDE[nbm]
    load_pos = {st * j + (st * w) // 4: j for j in range(8)} if loads else {}
    assert not loads or (len(load_pos) == 8 and max(load_pos) < n - 16)
    out = []
    adv = (advance() if loads else []) + tail
    assert len(adv) <= 15
    i = 0
    for q in range(2):
        for bm in range(nbm):
            # column blocks back and forth, so that from one MFMA to the next only one of the two fragment operands
            # changes (the row block's fragment stays for four MFMAs, and at the turn the column block's stays)
            for bn in (range(4) if (bm + q * nbm) % 2 == 0 else range(3, -1, -1)):
                out.append(f"v_mfma_f32_16x16x32_bf16 {acc(bm, bn)}, {fb(q, bn)}, {fa(q, bm)}, {acc(bm, bn)}")
                if i in load_pos:
                    out += load(load_pos[i])
                if n - 16 <= i < n - 1 and adv:
                    out.append(adv.pop(0))
                i += 1
    assert not adv
    return out


def group0(w, layout, nbm=8):
    """Waves 0-3: read phase of K step u, barrier, MFMA phase of u, barrier.  Tile 2u+4 is loaded during the MFMA phase
    of step u; the last two steps have no tile left to load and run a copy of the step without loads (its wait is for
    everything still in flight: the first tile of the last step).  nbm < 8: the variant for an output tile whose rows
    end inside this group's half (rows 0-127): only the first nbm 16-row blocks are read and multiplied."""
    s = ["s_cmp_le_u32 s45, 2", "s_cbranch_scc1 L0_drain_%="]
    s += ["L0_top_%=:"] + mem_phase(layout, nbm) + ["s_add_u32 s49, s44, s52", "s_waitcnt lgkmcnt(0)", "s_barrier"]
    s += mfma_phase(w, ["s_sub_u32 s45, s45, 1", "s_waitcnt vmcnt(8)"], nbm)
    s += ["s_barrier", "s_cmp_gt_u32 s45, 2", "s_cbranch_scc1 L0_top_%="]
    s += ["L0_drain_%=:"] + mem_phase(layout, nbm) + ["s_waitcnt lgkmcnt(0)", "s_barrier"]
    s += mfma_phase(w, ["s_sub_u32 s45, s45, 1", "s_waitcnt vmcnt(0)"], nbm, loads=False)
    s += ["s_barrier", "s_cmp_lg_u32 s45, 0", "s_cbranch_scc1 L0_drain_%=", "s_nop 15", "s_nop 15"]
    return s


def group1(w, layout, nbm=8):
    """Waves 4-7: one phase behind group 0 (extra barrier first); loads tile 2u+5 in the MFMA phase of step u, nothing in
    the last two steps.  nbm < 8: the variant for an output tile whose valid rows end inside this group's half (rows
    128-255): only the first nbm 16-row blocks are read and multiplied."""
    s = ["s_barrier", "s_cmp_le_u32 s45, 2", "s_cbranch_scc1 L1_drain_%="]
    s += ["L1_top_%=:"] + mem_phase(layout, nbm) + ["s_add_u32 s49, s44, s52", "s_waitcnt vmcnt(0) lgkmcnt(0)", "s_barrier"]
    s += mfma_phase(w, ["s_sub_u32 s45, s45, 1"], nbm)
    s += ["s_barrier", "s_cmp_gt_u32 s45, 2", "s_cbranch_scc1 L1_top_%="]
    s += ["L1_drain_%=:"] + mem_phase(layout, nbm) + ["s_waitcnt vmcnt(0) lgkmcnt(0)", "s_barrier"]
    s += mfma_phase(w, ["s_sub_u32 s45, s45, 1"], nbm, loads=False)
    s += ["s_cmp_lg_u32 s45, 0", "s_cbranch_scc0 L1_end_%=",
          "s_barrier", "s_branch L1_drain_%=", "L1_end_%=:", "s_nop 15", "s_nop 15"]
    return s


G0_SHORT = (4, 6)            # row blocks of the short variants of each group
G1_SHORT = (4, 5, 6, 7)


def macro(name, lines):
    return f"#define {name} \\\n" + " \\\n".join('  "' + l + '\\n\\t"' for l in lines)


def main():
    clob = ", ".join(f'"v{i}"' for i in range(128, 231))
    out = ["// Generated by gen_mainloop.py -- do not edit by hand.", "#pragma once"]
    for layout in range(4):
        for w in range(4):
            out.append(macro(f"GSPMD_MAINLOOP_L{layout}_G0_W{w}", group0(w, layout)))
            for nbm in G0_SHORT:
                out.append(macro(f"GSPMD_MAINLOOP_L{layout}_G0R{nbm}_W{w}", group0(w, layout, nbm)))
            out.append(macro(f"GSPMD_MAINLOOP_L{layout}_G1_W{w}", group1(w, layout)))
            for nbm in G1_SHORT:
                out.append(macro(f"GSPMD_MAINLOOP_L{layout}_G1R{nbm}_W{w}", group1(w, layout, nbm)))
    out.append(f'#define GSPMD_MAINLOOP_CLOBBERS {clob}, "s48", "s49", "s50", "s51", "m0", "scc", "vcc", "memory"')
    sys.stdout.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
