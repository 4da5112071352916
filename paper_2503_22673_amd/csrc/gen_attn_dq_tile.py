#!/usr/bin/env python3
"""Writes attn_dq_tile.inc: one (64 queries x 64 keys) tile step of attn_bwd_dq3_mfma (attention_mfma.hip, head_dim
128) as one inline-asm block.  Run by hand after a change (python gen_attn_dq_tile.py); the generated file is
committed.  Same construction as gen_attn_dkv_tile.py (one wave per SIMD, everything behind the MFMAs, waits derived by
replaying the sequence); what differs:

  * a lane owns two queries (query blocks 0 and 1 of the wave's 64), so every fragment read from LDS feeds two MFMAs
    and the per-query values (lse, delta, mask bounds) are plain per-lane registers;
  * 96 v_mfma_f32_32x32x16_bf16 per step:
      slots  0..31  S(qb, kb) = K Q^T for the key blocks kb = 0, 1: per slice one K fragment, two MFMAs
      slots 32..63  dP(qb, kb) = V dO^T likewise
      slots 64..95  dQ^T(qb) += K^T dS^T: per 16-key chunk x and column block cb one fragment, two MFMAs
  * K and V sit in LDS once, row major [64 keys][128], position of chunk c of row r = c ^ f(r) as in the dK / dV kernel;
    the last product reads K through ds_read_b64_tr_b16, so no token-major copy of K exists;
  * eight loads per wave and tile (four kilobytes of K, four of V) of the tile two steps ahead.

The block dispatches on %51: bits 0..1 = 1 every query sees every key, 2 mask by the lane's queries; bit 2 = issue the
loads.

Operands: %0..%7 dQ^T blocks (query block, column block) (accumulation registers); %8..%23 Q fragments, %24..%39 dO
fragments (query block, slice) (accumulation registers, read as B operands); %40 LDS address of this lane's row of the K
tile of the stage (V 16 KB behind), chunk h ^ swizzle; %41 LDS address of this lane's corner of the 4 x 16 patch for
the transposing reads; %42 sl2 (scalar); %43, %44 -lse log2 e of the lane's two queries; %45, %46 their delta;
%47, %48 = k0 + 4 h - segment start of the query, %49, %50 = query - segment start (a key is seen when its offset from
the segment start is at most that); %52, %53 addresses of the first K / V row of the tile to load (scalar pairs),
%54 bytes between the row groups of consecutive loads, %55 this lane's byte offset in the first load, %56 LDS address of
this wave's first kilobyte of the stage to fill.
Fixed registers (clobbered): v45 load offset, v46 temp, v47 -inf, v[48:55] patch addresses per column block (rows
0..3 / 8..11 of a chunk), v[56:63] row addresses per slice, v[64:95] fragments, v[96:127] dS operands (query block,
chunk), v[128:191] S (query block, key block), v[192:255] dP; s[80:83] running load addresses, s86 the caller's m0.
"""
import os

OP_DQ, OP_QF, OP_DOF, OP_AR, OP_AT, OP_SL2, OP_NL, OP_DL, OP_TB, OP_LIM, OP_MODE, OP_GK, OP_GV, OP_STR, OP_VOFF, OP_M0T = \
    0, 8, 24, 40, 41, 42, 43, 45, 47, 49, 51, 52, 53, 54, 55, 56
CAP = int(os.environ.get('ATTN_DQ_CAP', '6'))     # vector-ALU issue units behind one MFMA (v_exp counts 2)
CAP_MASKED = 12
NS = 96
LOAD_SLOTS = [5, 17, 29, 41, 53, 65, 77, 89]


def tup(base, n): return "v[%d:%d]" % (base, base + n - 1)
def S(qb, kb, e): return "v%d" % (128 + 16 * (2 * qb + kb) + e)
def DP(qb, kb, e): return "v%d" % (192 + 16 * (2 * qb + kb) + e)
def DSB(qb, x, j): return "v%d" % (96 + 16 * qb + 4 * x + j)
def F(i): return tup(64 + 4 * i, 4)


def frag_list():
    """48 fragments, each feeding the two MFMAs (query blocks 0, 1) of slots 2 f, 2 f + 1:
    (reads, [(dst text or operand, b operand, first)] per query block)"""
    L = []
    for kb in range(2):
        for ks in range(8):
            reads = [("ds_read_b128 %%s, v%d offset:%d" % (56 + ks, kb * 8192), 0, 4)]
            L.append((reads, [(tup(128 + 16 * (2 * qb + kb), 16), "%%%d" % (OP_QF + 8 * qb + ks), ks == 0) for qb in range(2)]))
    for kb in range(2):
        for ks in range(8):
            reads = [("ds_read_b128 %%s, v%d offset:%d" % (56 + ks, 16384 + kb * 8192), 0, 4)]
            L.append((reads, [(tup(192 + 16 * (2 * qb + kb), 16), "%%%d" % (OP_DOF + 8 * qb + ks), ks == 0) for qb in range(2)]))
    for x in range(4):
        for cb in range(4):
            reads = [("ds_read_b64_tr_b16 %%s, v%d offset:%d" % (48 + cb, x * 4096), 0, 2),
                     ("ds_read_b64_tr_b16 %%s, v%d offset:%d" % (52 + cb, x * 4096 + 2048), 2, 2)]
            L.append((reads, [("%%%d" % (OP_DQ + 4 * qb + cb), tup(96 + 16 * qb + 4 * x, 4), False) for qb in range(2)]))
    assert len(L) == 48
    return L


def groups(masked):
    G = []
    for kb in range(2):
        s_ready = 20 + 16 * kb           # the S chains of key block kb end at slots 14, 15 + 16 kb
        d_ready = 52 + 16 * kb           # the dP chains at 46, 47 + 16 kb
        for qb in range(2):
            for b4 in range(4):
                ins = []
                for i in range(4):
                    e = 4 * b4 + i
                    if masked:
                        c = kb * 32 + 8 * (e >> 2) + (e & 3)
                        ins += [("v_add_u32 v46, %d, %%%d" % (c, OP_TB + qb), 1), ("v_cmp_le_u32 vcc, v46, %%%d" % (OP_LIM + qb), 1),
                                ("v_cndmask_b32 %s, v47, %s, vcc" % (S(qb, kb, e), S(qb, kb, e)), 1)]
                for i in range(4):
                    e = 4 * b4 + i
                    ins.append(("v_fma_f32 %s, %s, %%%d, %%%d" % (S(qb, kb, e), S(qb, kb, e), OP_SL2, OP_NL + qb), 1))
                for i in range(4):
                    e = 4 * b4 + i
                    ins.append(("v_exp_f32 %s, %s" % (S(qb, kb, e), S(qb, kb, e)), 2))
                x = 2 * kb + (b4 >> 1)
                G.append(dict(name="E%d%d%d" % (kb, qb, b4), ready=s_ready, deadline=64 + 8 * x, ins=ins))
        for qb in range(2):
            for sl in range(2):
                x = 2 * kb + sl
                ins = []
                for e in range(8 * sl, 8 * sl + 8):
                    ins.append(("v_sub_f32 %s, %s, %%%d" % (DP(qb, kb, e), DP(qb, kb, e), OP_DL + qb), 1))
                for e in range(8 * sl, 8 * sl + 8):
                    ins.append(("v_mul_f32 %s, %s, %s" % (DP(qb, kb, e), S(qb, kb, e), DP(qb, kb, e)), 1))
                for j in range(4):
                    ins.append(("v_cvt_pk_bf16_f32 %s, %s, %s" % (DSB(qb, x, j), DP(qb, kb, 8 * sl + 2 * j), DP(qb, kb, 8 * sl + 2 * j + 1)), 1))
                G.append(dict(name="D%d%d%d" % (kb, qb, sl), ready=d_ready, deadline=64 + 8 * x, ins=ins))
    return G


def schedule(masked, cap):
    """slot -> vector instructions.  The list order of the groups is a valid program order (E before D of the same
    elements); earliest deadline first with ties in list order keeps it, because a D group never has an earlier
    deadline than the E groups of its elements and becomes ready later."""
    G = groups(masked)
    order = {g["name"]: i for i, g in enumerate(G)}
    slots = [[] for _ in range(NS)]
    pending = list(G)
    cur, left = None, []
    for slot in range(NS):
        room = cap
        while room > 0:
            if cur is None:
                ready = [g for g in pending if g["ready"] <= slot]
                if not ready:
                    break
                cur = min(ready, key=lambda g: (g["deadline"], order[g["name"]]))
                pending.remove(cur)
                left = list(cur["ins"])
            text, cost = left[0]
            if cost > room and room < cap:
                break
            slots[slot].append(text)
            room -= cost
            left.pop(0)
            if not left:
                assert slot < cur["deadline"], ("deadline missed", cur["name"], slot, cur["deadline"])
                cur = None
    assert not pending and cur is None, [g["name"] for g in pending]
    return slots


def load_ops(k):
    """the k-th load of the tile two steps ahead: K row groups 0..3, V row groups 0..3"""
    which, i = k // 4, k % 4
    base = "s[80:81]" if which == 0 else "s[82:83]"
    lo, hi = ("s80", "s81") if which == 0 else ("s82", "s83")
    ops = ["s_add_u32 m0, %%%d, %d" % (OP_M0T, which * 16384 + i * 1024),
           "v_xor_b32 v45, %d, %%%d" % (16 * (((i & 1) << 1) | (i >> 1)), OP_VOFF),     # the row group's part of the swizzle
           "global_load_lds_dwordx4 v45, %s" % base]
    if i < 3:
        ops += ["s_add_u32 %s, %s, %%%d" % (lo, lo, OP_STR), "s_addc_u32 %s, %s, 0" % (hi, hi)]
    return ops


def load_prologue():
    return ["s_mov_b32 s86, m0", "s_mov_b64 s[80:81], %%%d" % OP_GK, "s_mov_b64 s[82:83], %%%d" % OP_GV]


def emit(masked, loads):
    FL = frag_list()
    vslots = schedule(masked, CAP_MASKED if masked else CAP)
    out = []
    lds_issued = 0
    lds_done = 0
    src = {}
    last_exp = {}
    n_ins = [0]

    def put(t):
        out.append(t)
        n_ins[0] += 1

    def wait_lds(idx):
        nonlocal lds_done
        if idx <= lds_done:
            return
        younger = lds_issued - idx
        assert younger <= 15, ("lgkmcnt cannot express", younger)
        put("s_waitcnt lgkmcnt(%d)" % younger)
        lds_done = idx

    def frag_reads(f):
        nonlocal lds_issued
        base = 64 + 4 * (f % 8)
        for text, off, n in FL[f][0]:
            lds_issued += 1
            src["F%d" % (f % 8)] = lds_issued
            put(text % tup(base + off, n))

    def valu(text):
        toks = text.replace(",", " ").split()
        regs = [t for t in toks[1:] if t.startswith("v") and t[1:].isdigit()]
        if not toks[0].startswith("v_exp"):
            for r in regs[1:]:
                if r in last_exp and n_ins[0] - last_exp[r] < 2:
                    put("s_nop 0")
        put(text)
        if toks[0].startswith("v_exp"):
            last_exp[regs[0]] = n_ins[0]
        elif regs and regs[0] in last_exp:
            del last_exp[regs[0]]

    put("s_nop 1")
    if loads:
        for t in load_prologue():
            put(t)
    if masked:
        put("v_mov_b32 v47, 0xff800000")
    for ks in range(8):                       # slice addresses: the swizzle is an XOR on the chunk bits, so is the slice
        put("v_xor_b32 v%d, %d, %%%d" % (56 + ks, 32 * ks, OP_AR))
        if ks < 4:
            frag_reads(ks)
    for cb in range(4):                       # patch addresses: column block cb, rows 0..3 and 8..11 of a key chunk
        put("v_xor_b32 v%d, %d, %%%d" % (48 + cb, 64 * cb, OP_AT))
        put("v_xor_b32 v%d, %d, %%%d" % (52 + cb, (64 * cb) ^ 16, OP_AT))
    for m in range(NS):
        f, qb = m // 2, m % 2
        wait_lds(src["F%d" % (f % 8)])
        d, b, first = FL[f][1][qb]
        put("v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (d, F(f % 8), b, "0" if first else d))
        if qb == 1 and 4 <= f + 3 < 48:       # the fragment three ahead; its registers were last read by the MFMAs of fragment f - 5
            frag_reads(f + 3)
        if loads and m in LOAD_SLOTS:
            for t in load_ops(LOAD_SLOTS.index(m)):
                put(t)
        for text in vslots[m]:
            valu(text)
    if loads:
        put("s_mov_b32 m0, s86")
    return out


def main(out_path=None):
    lines = []
    for mode, body in ((1, emit(False, False)), (2, emit(True, False)), (5, emit(False, True)), (6, emit(True, True))):
        lines += ["s_cmp_eq_u32 %%%d, %d" % (OP_MODE, mode), "s_cbranch_scc0 L_dq_not%d_%%=" % mode] + body + \
                 ["s_branch L_dq_end_%=", "L_dq_not%d_%%=:" % mode]
    lines.append("L_dq_end_%=:")
    out = out_path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_dq_tile.inc")
    with open(out, "w") as f:
        f.write("// Generated by gen_attn_dq_tile.py -- do not edit.  One tile step of attn_bwd_dq3_mfma.\n")
        f.write("#define ATTN_DQ_TILE_ASM \\\n")
        for ln in lines:
            f.write('  "%s\\n" \\\n' % ln)
        f.write('  ""\n')
        vregs = ", ".join('"v%d"' % i for i in range(45, 256))
        f.write("#define ATTN_DQ_TILE_CLOBBERS %s, \"s80\", \"s81\", \"s82\", \"s83\", \"s86\", \"vcc\", \"scc\", \"memory\"\n" % vregs)
    print("wrote", out, len(lines), "instructions")


if __name__ == "__main__":
    import sys
    main(sys.argv[1] if len(sys.argv) > 1 else None)
