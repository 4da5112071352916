#!/usr/bin/env python3
"""Writes gemm_rs_loop.inc: the hand-scheduled main loop of gemm_mfma_rs_kernel (gemm.hip) as one inline-asm
block.  Run by hand after a change (python gen_gemm_rs_loop.py); the generated file is committed.

One K step (64 wide) of one wave (a 128 x 128 block of a 256 x 256 tile, four waves, one per SIMD) is 64
v_mfma_f32_32x32x16_bf16 on 16 accumulators, and behind every MFMA rides one other memory instruction, at a
uniform rate: per four MFMAs two LDS fragment reads, one LDS store and one global load (a CU's vector memory path
takes 64 bytes a clock: four waves that load at the same time must not ask for more than one 1 KB load per four
MFMAs each, or they stall in the issue of the load and the matrix pipe idles with them).

Pipeline of a tile t: its 16 loads (A rows 0..7, B rows 0..7 of this wave's share) are issued at slots 4n + 3 of step
t - 3 into register stage (t & 1); register n is stored to LDS stage (t & 1) 111 slots later (n < 4: slots 50 .. 62
of step t - 2 ... see below), i.e. a load has 1.7 K steps to arrive; the store sits 17 slots before the next load
into the same registers.  The LDS stage of tile t may be written from the barrier of step t - 2 (slot 49: everyone
has read tile t - 2) to the barrier of step t - 1, after which everyone reads tile t.  In steady state exactly 27
loads are younger than the one a store waits for (vmcnt(27)); LDS operations complete in order, so fragment
waits are lgkmcnt(k) with k the number of LDS operations issued after the read in question.  The waits are
computed below by replaying the instruction sequence.

Register map (vector): v[0:63], v[64:127] register stages (A loads 0..7, then B loads 0..7, 4 registers each);
v[128:159], v[160:191] fragment sets (A blocks 0..3, then B blocks 0..3); v[192:195] / v[196:199] LDS read
addresses of A / B per 16-wide slice; v200..v203 LDS store addresses (A even / odd load, B even / odd load);
v[206:209] per-lane byte offsets of A and B rows in segment 0 and 1; (v204, v205), (v210, v211) those of the
tile being loaded in even / odd steps.  Scalar: s[40:47] operand bases of both segments, s[48:51] their 8-row
strides, s52 nt0, s53 nt, s54 nt - 1, s67 step, s66 / s68 .. s73 temps; running bases and strides of the loads:
s[60:65] in even steps, s[74:79] in odd steps.
"""
import os

OP_SCRATCH, OP_A0, OP_B0, OP_A1, OP_B1, OP_SA0, OP_SB0, OP_SA1, OP_SB1, OP_NT0, OP_NT = range(16, 27)
A_STAGE = 32768                         # LDS bytes: A stages at 0 / 32768, B stages at 65536 / 98304 (inside the addresses)
READ_ORDER = [("a", 0), ("b", 0), ("b", 1), ("b", 2), ("b", 3), ("a", 1), ("a", 2), ("a", 3)]
READ_SLOTS = [0, 1, 2, 3, 4, 5, 6, 7]                    # within slices 0..2: fragments of the next slice
READ_SLOTS_LAST = [50, 51, 52, 53, 54, 55, 56, 57]      # slice 3: after the barrier, fragments of the next tile
BARRIER_SLOT = 49
DIST = 2          # a step loads tile it + 1 + DIST: 2 = as early as the register stages allow (1.7 steps in flight), 1 = one step later
STORE_SLOTS = [58, 60, 62, 63, 8, 10, 12, 14, 24, 26, 28, 30, 40, 42, 44, 46]   # register n; the first four belong to the previous step
LOAD_SLOTS = [9, 11, 13, 15, 25, 27, 29, 31, 41, 43, 45, 47, 48, 49, 59, 61]    # register n


def frag(setno, which, idx):
    base = 128 + 32 * setno + (0 if which == "a" else 16) + 4 * idx
    return "v[%d:%d]" % (base, base + 3)


def stage_reg(stage, n):
    base = 64 * stage + 4 * n           # n < 8: A loads, n >= 8: B loads
    return "v[%d:%d]" % (base, base + 3)


def scal(P):
    """(A base pair, B base pair, A stride, B stride, A offset vgpr, B offset vgpr) of the loads issued in a step of parity P"""
    return (("s60", "s61", "s62", "s63", "s64", "s65", "v204", "v205") if P == 0 else
            ("s74", "s75", "s76", "s77", "s78", "s79", "v210", "v211"))


def text_read(setno, lds_stage, ks, which, idx):
    return "ds_read_b128 %s, v%d offset:%d" % (frag(setno, which, idx), (192 if which == "a" else 196) + ks,
                                                lds_stage * A_STAGE + idx * 4096)


def text_store(reg_stage, lds_stage, n):
    which, i = ("a", n) if n < 8 else ("b", n - 8)
    addr = (200 if which == "a" else 202) + (i & 1)
    return "ds_write_b128 v%d, %s offset:%d" % (addr, stage_reg(reg_stage, n), lds_stage * A_STAGE + i * 1024)


def text_load(reg_stage, n, P):
    alo, ahi, blo, bhi, sa, sb, va, vb = scal(P)
    if n < 8:
        return ["global_load_dwordx4 %s, %s, s[%s:%s]" % (stage_reg(reg_stage, n), va, alo[1:], ahi[1:]),
                "s_add_u32 %s, %s, %s" % (alo, alo, sa), "s_addc_u32 %s, %s, 0" % (ahi, ahi)]
    return ["global_load_dwordx4 %s, %s, s[%s:%s]" % (stage_reg(reg_stage, n), vb, blo[1:], bhi[1:]),
            "s_add_u32 %s, %s, %s" % (blo, blo, sb), "s_addc_u32 %s, %s, 0" % (bhi, bhi)]


def tile_bases(P):
    """s66 = tile to load (clamped here to the last one); sets the running bases, strides and offsets of parity P"""
    alo, ahi, blo, bhi, sa, sb, va, vb = scal(P)
    return ["s_min_i32 s66, s66, s54",
            "s_cmp_lt_i32 s66, s52",                      # scc: the tile lies in segment 0
            "s_cselect_b32 s69, 0, s52",
            "s_cselect_b64 s[70:71], s[40:41], s[44:45]",
            "s_cselect_b64 s[72:73], s[42:43], s[46:47]",
            "s_cselect_b32 %s, s48, s50" % sa,
            "s_cselect_b32 %s, s49, s51" % sb,
            "s_cselect_b64 vcc, -1, 0",
            "s_sub_i32 s68, s66, s69",
            "s_lshl_b32 s68, s68, 7",                      # 64 bf16 = 128 bytes per K step
            "s_add_u32 %s, s70, s68" % alo, "s_addc_u32 %s, s71, 0" % ahi,
            "s_add_u32 %s, s72, s68" % blo, "s_addc_u32 %s, s73, 0" % bhi,
            "v_cndmask_b32 %s, v208, v206, vcc" % va,
            "v_cndmask_b32 %s, v209, v207, vcc" % vb]


def step_ops(P):
    """Operations of one step of parity P as a list of 64 slots; slot g = [MFMA, then the operations behind it].
    Tile `it` is read from LDS stage P; tile it+1 goes register stage Q -> LDS stage Q (registers 4..15; 0..3 went in
    the previous step), tile it+2 register stage P -> LDS stage P (registers 0..3, after the barrier), tile it+3 is
    loaded into register stage Q."""
    Q = P ^ 1
    slots = [[] for _ in range(64)]
    for s in range(4):
        for m in range(16):
            slots[16 * s + m].append(("mfma", s & 1, m))
    for s in range(3):                                     # fragments of slice s+1 of this tile
        for k, (which, idx) in enumerate(READ_ORDER):
            slots[16 * s + READ_SLOTS[k]].append(("read", (s + 1) & 1, P, s + 1, which, idx))
    slots[BARRIER_SLOT].append(("barrier",))
    for k, (which, idx) in enumerate(READ_ORDER):          # fragments of slice 0 of the next tile
        slots[READ_SLOTS_LAST[k]].append(("read", 0, Q, 0, which, idx))
    slots[BARRIER_SLOT].remove(("barrier",))
    for n in range(16):
        slots[LOAD_SLOTS[n]].append(("load", Q if DIST == 2 else P, n, P))
    slots[BARRIER_SLOT].append(("barrier",))
    for n in range(4, 16):
        slots[STORE_SLOTS[n]].append(("store", Q, Q, n))
    for n in range(4):
        slots[STORE_SLOTS[n]].append(("store", P, P, n))
    # scalar work for the next step's loads (tile it+4, other scalar set), spread behind the first MFMAs
    # (the run from the compare to the last select depends on scc, which the loads' address updates overwrite: one slot)
    tb = ["s_add_i32 s66, s67, %d" % (2 + DIST)] + tile_bases(Q)
    for slot, lo, hi in ((16, 0, 9), (18, 9, 11), (20, 11, 13), (22, 13, 15), (24, 15, 17)):
        slots[slot].append(("scalar", tb[lo:hi]))
    return slots


def emit_steps(e):
    """Replays three steps (parity 0, 1, 0) to find every wait, and emits the last two (parity 1 first is wrong
    for the loop, so the order emitted is: the third step's text for parity 0, the second's for parity 1)."""
    seq = []                                               # (step index, op)
    for k, P in enumerate((0, 1, 0, 1)):
        for g, ops in enumerate(step_ops(P)):
            for op in ops:
                seq.append((k, g, op))
    out = {2: [], 3: []}
    lds_issued = 0                                         # running counts of LDS operations / loads issued
    vm_issued = 0
    frag_src = {}                                          # fragment register -> index (in LDS order) of the read that fills it
    store_idx = {}                                         # (reg stage, n) -> LDS index of its last store
    load_idx = {}                                          # (reg stage, n) -> VMEM index of its last load
    lds_done = 0                                           # every LDS operation with index <= lds_done is known complete
    vm_done = 0
    for k, g, op in seq:
        em = out.get(k)
        def wait_lds(idx):
            nonlocal lds_done
            if idx <= lds_done:
                return
            younger = lds_issued - idx
            assert younger <= 15, ("lgkmcnt cannot express", younger, k, g, op)
            if em is not None:
                em.append("s_waitcnt lgkmcnt(%d)" % younger)
            lds_done = idx
        def wait_vm(idx):
            nonlocal vm_done
            if idx <= vm_done:
                return
            younger = vm_issued - idx
            assert younger <= 63
            if em is not None:
                em.append("s_waitcnt vmcnt(%d)" % younger)
            vm_done = idx
        kind = op[0]
        if kind == "mfma":
            _, setno, m = op
            i, j = m // 4, m % 4
            for key in ((setno, "a", i), (setno, "b", j)):
                if key in frag_src:
                    wait_lds(frag_src[key])
            if em is not None:
                acc = "%%%d" % (4 * i + j)
                # operands swapped (B fragment first): the result block comes out transposed, i.e. a lane owns one ROW of
                # the 32 x 32 block of C and four consecutive columns per accumulator quad, which the epilogue stores 8 bytes at a time
                em.append("v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (acc, frag(setno, "b", j), frag(setno, "a", i), acc))
        elif kind == "read":
            _, setno, lds_stage, ks, which, idx = op
            lds_issued += 1
            frag_src[(setno, which, idx)] = lds_issued
            if em is not None:
                em.append(text_read(setno, lds_stage, ks, which, idx))
        elif kind == "store":
            _, reg_stage, lds_stage, n = op
            if (reg_stage, n) in load_idx:
                wait_vm(load_idx[(reg_stage, n)])
            lds_issued += 1
            store_idx[(reg_stage, n)] = lds_issued
            if em is not None:
                em.append(text_store(reg_stage, lds_stage, n))
        elif kind == "load":
            _, reg_stage, n, P = op
            if (reg_stage, n) in store_idx:                # the store has read these registers
                if lds_issued - store_idx[(reg_stage, n)] <= 15:
                    wait_lds(store_idx[(reg_stage, n)])
                else:
                    assert store_idx[(reg_stage, n)] <= lds_done, "a store 16 LDS operations back is not known complete"
            vm_issued += 1
            load_idx[(reg_stage, n)] = vm_issued
            if em is not None:
                em.extend(text_load(reg_stage, n, P))
        elif kind == "barrier":
            wait_lds(lds_issued)                           # this wave's stores are in LDS and its reads of the tile are done
            if em is not None:
                em.append("s_barrier")
        elif kind == "scalar":
            if em is not None:
                em.extend(op[1])
    return out[2], out[3]


class Emitter:
    def __init__(self):
        self.lines = []

    def __call__(self, s):
        if isinstance(s, list):
            self.lines.extend(s)
        else:
            self.lines.append(s)


def main(out_path=None):
    e = Emitter()
    # ---- set-up: per-lane values from the LDS scratch line of this lane, scalars from the operands
    e("ds_read_b128 v[192:195], %%%d" % OP_SCRATCH)
    e("ds_read_b128 v[196:199], %%%d offset:16" % OP_SCRATCH)
    e("ds_read_b128 v[200:203], %%%d offset:32" % OP_SCRATCH)
    e("ds_read_b128 v[206:209], %%%d offset:48" % OP_SCRATCH)
    for dst, op in (("s[40:41]", OP_A0), ("s[42:43]", OP_B0), ("s[44:45]", OP_A1), ("s[46:47]", OP_B1)):
        e("s_mov_b64 %s, %%%d" % (dst, op))
    for dst, op in (("s48", OP_SA0), ("s49", OP_SB0), ("s50", OP_SA1), ("s51", OP_SB1), ("s52", OP_NT0), ("s53", OP_NT)):
        e("s_mov_b32 %s, %%%d" % (dst, op))
    e("s_sub_i32 s54, s53, 1")
    e("s_waitcnt lgkmcnt(0)")
    # ---- prologue: the state the loop expects at step 0 -- tile 0 in LDS stage 0, registers 0..3 of tile 1 in LDS
    # stage 1, registers 4..15 of tile 1 and all of tile 2 in flight in that order, slice 0 of tile 0 in fragment set 0,
    # the scalar set of even steps pointing at tile 3
    for t, stage in ((0, 0), (1, 1)):
        e("s_mov_b32 s66, %d" % t)
        e(tile_bases(0))
        for n in range(16):
            e(text_load(stage, n, 0))
    e("s_waitcnt vmcnt(16)")
    for n in range(16):
        e(text_store(0, 0, n))
    e("s_waitcnt lgkmcnt(0)")                      # the stores have read their registers
    if DIST == 2:
        e("s_mov_b32 s66, 2")
        e(tile_bases(0))
        for n in range(16):
            e(text_load(0, n, 0))
        e("s_waitcnt vmcnt(28)")
    else:
        e("s_waitcnt vmcnt(12)")
    for n in range(4):
        e(text_store(1, 1, n))
    e("s_waitcnt lgkmcnt(0)")
    e("s_barrier")
    for which, idx in READ_ORDER:
        e(text_read(0, 0, 0, which, idx))
    e("s_mov_b32 s66, %d" % (1 + DIST))
    e(tile_bases(0))
    e("s_mov_b32 s67, 0")
    e("s_waitcnt lgkmcnt(0)")
    # ---- main loop, two steps per trip
    even, odd = emit_steps(e)
    e("L_rs_loop_%=:")
    e(even)
    e("s_add_i32 s67, s67, 1")
    e("s_cmp_ge_i32 s67, s53")
    e("s_cbranch_scc1 L_rs_end_%=")
    e(odd)
    e("s_add_i32 s67, s67, 1")
    e("s_cmp_lt_i32 s67, s53")
    e("s_cbranch_scc1 L_rs_loop_%=")
    e("L_rs_end_%=:")
    # the re-requested tiles must land before their registers are reused; the last MFMAs must have written
    e("s_waitcnt vmcnt(0) lgkmcnt(0)")
    e("s_nop 15")
    e("s_nop 15")

    out = out_path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "gemm_rs_loop.inc")
    with open(out, "w") as f:
        f.write("// Generated by gen_gemm_rs_loop.py -- do not edit.  Main loop of gemm_mfma_rs_kernel.\n")
        f.write("#define GEMM_RS_LOOP_ASM \\\n")
        for ln in e.lines:
            f.write('  "%s\\n" \\\n' % ln)
        f.write('  ""\n')
        vregs = ", ".join('"v%d"' % i for i in range(212))
        sregs = ", ".join('"s%d"' % i for i in range(40, 80))
        f.write("#define GEMM_RS_LOOP_CLOBBERS %s, %s, \"vcc\", \"scc\", \"memory\"\n" % (vregs, sregs))
    print("wrote", out, len(e.lines), "instructions")


if __name__ == "__main__":
    import sys
    main(sys.argv[1] if len(sys.argv) > 1 else None)
