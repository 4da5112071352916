#!/usr/bin/env python3
"""Writes attn_dkv_tile.inc: one (32 keys x 64 queries) tile step of attn_bwd_dkv3_mfma (attention_mfma.hip, head_dim
128) as one inline-asm block.  Run by hand after a change (python gen_attn_dkv_tile.py); the generated file is
committed.

The wave runs alone on its SIMD (both halves of the register file), so nothing but its own instruction order can keep
the matrix pipe busy while the vector ALU works and the next tiles arrive.  A tile step is 64
v_mfma_f32_32x32x16_bf16:

  slots  0..15  S0, then dP0, over the 8 slices of head_dim (queries 0..31 of the tile)
  slots 16..31  S1, then dP1                                 (queries 32..63)
  slots 32..39  dV += dO^T P^T   for the query chunks 0, 1 (of 16) x 4 column blocks
  slots 40..47  dK += Q^T  dS^T  for the query chunks 0, 1
  slots 48..55  dV, chunks 2, 3
  slots 56..63  dK, chunks 2, 3

and behind every MFMA ride the other instructions:

  * the LDS reads of the fragment six MFMAs ahead (eight rotating fragment registers).  Q and dO sit in LDS once, row
    major [64 queries][128]; the 16-byte chunk c of row r sits at position c ^ f(r), f = the low four bits of r in the
    order (1, 0, 2, 3): rows r .. r + 3 differ in the top two bits of the position, r and r + 4 in bit 1, r and r + 8 in
    bit 0, which keeps the row reads (16 rows, one chunk) and the patch reads below (4 or 8 rows, 2 to 4 chunks) off each
    other's banks.  S and dP read them as rows
    (ds_read_b128).  dV and dK contract over the queries and need them transposed: ds_read_b64_tr_b16 hands a lane,
    for its column, the elements of four consecutive rows (the 16 lanes of a block point at a 4 row x 16 column
    patch, four columns each), so a fragment is two such reads and no transposed copy of Q or dO exists anywhere;
  * the reads of the lse / delta values;
  * the vector work -- P = exp2(S sl2 - lse log2 e), dS = P (dP - delta), both rounded to bf16 as B operands -- placed by
    an earliest-deadline list scheduler between the slot where its inputs are complete (four MFMAs after the last
    one of the chain: the hardware does not interlock a vector read of a matrix result) and the slot of the MFMA that
    consumes it;
  * the nine loads (global -> LDS, 1 KB each) of this wave's share of the tile two steps ahead, one every seven
    slots: issued in a burst they would hold the wave in the issue of the loads, because a CU's path into LDS takes
    about 40 bytes a clock.

LDS operations complete in order, so a wait is lgkmcnt(k) with k the number of LDS operations issued after the one in
question; the waits are derived by replaying the sequence.  The transcendental unit forwards late: a
non-transcendental read of a v_exp result keeps a distance of two instructions.

The block dispatches on %30: bits 0..1 = 0 no query of the tile sees a key of this wave, 1 every query sees every
key, 2 mask by the lane's key; bit 2 = issue the loads.

Operands: %0..%3 dK^T blocks, %4..%7 dV^T blocks (accumulation registers); %8..%15 K fragments, %16..%23 V fragments
of this wave's keys (accumulation registers, read as B operands); %24 LDS address of this lane's row of the Q tile of
the stage (dO 16 KB behind), chunk h ^ swizzle; %25 LDS address of this lane's corner of the 4 x 16 patch for the
transposing reads (rows 4 h + .., column block 0); %26 address of the stage's lse values + 16 h (delta 256 B behind);
%27 sl2 (scalar); %28 = t0 + 4 h - u, %29 = number of queries from u that see the key (0 for a lane without key);
%31, %32 addresses of the first Q / dO row of the tile to load (scalar pairs), %33, %34 bytes between the row groups
of consecutive loads, %35, %36 this lane's byte offsets in the first load, %37 LDS address of this wave's first
kilobyte of the stage to fill, %38 address of this lane's lse or delta value (vector pair), %39 its LDS address.
Fixed registers (clobbered): v92 load offset, v94 -inf, v95 temp, v[96:111] four rotating lse / delta quads,
v[112:119] Q / dO row addresses per slice, v[120:127] patch addresses per column block (rows 0..3 / 8..11 of a
chunk: an XOR of 16 and 2048 bytes on), v[128:159] S0 S1, v[160:191] dP0 dP1, v[192:207] P operands, v[208:223] dS operands, v[224:255]
fragments; s[80:83] running load addresses, s86 the caller's m0.
"""
import os

(OP_DK, OP_DV, OP_KF, OP_VF, OP_AR, OP_AT, OP_AL, OP_SL2, OP_TB, OP_LEN, OP_MODE,
 OP_GQ, OP_GD, OP_SQ, OP_SD, OP_VQ, OP_VD, OP_M0T, OP_VL, OP_M0L) = (0, 4, 8, 16, 24, 25, 26, 27, 28, 29, 30,
                                                                      31, 32, 33, 34, 35, 36, 37, 38, 39)
CAP = int(os.environ.get('ATTN_DKV_CAP', '6'))   # vector-ALU issue units behind one MFMA (v_exp counts 2): five plain ones behind an MFMA are free, the sixth costs 2 clocks, measured
CAP_MASKED = 10             # the masked form (tiles on the diagonal or a segment end) has 96 more instructions to place
NEG_LOG2E = "0xbfb8aa3b"
LOAD_SLOTS = [3, 10, 17, 24, 31, 38, 45, 52, 59]


def S(qb, e): return "v%d" % (128 + 16 * qb + e)
def DP(qb, e): return "v%d" % (160 + 16 * qb + e)
def tup(base, n): return "v[%d:%d]" % (base, base + n - 1)
def F(i): return tup(224 + 4 * i, 4)
def LQ(i, k): return "v%d" % (96 + 4 * i + k)
def BP(x, j): return "v%d" % (192 + 4 * x + j)
def BS(x, j): return "v%d" % (208 + 4 * x + j)


def mfma_list():
    """per slot: (kind, block index, fragment reads as (text with %s for the register, first register offset, registers), b operand, first of chain)"""
    L = []
    for qb in range(2):                       # whole chains one after the other: the vector work on S0 starts under dP0
        for ks in range(8):
            L.append(("S", qb, [("ds_read_b128 %%s, v%d offset:%d" % (112 + ks, qb * 8192), 0, 4)], "%%%d" % (OP_KF + ks), ks == 0))
        for ks in range(8):
            L.append(("dP", qb, [("ds_read_b128 %%s, v%d offset:%d" % (112 + ks, 16384 + qb * 8192), 0, 4)], "%%%d" % (OP_VF + ks), ks == 0))
    for half in range(2):
        for which in ("dV", "dK"):
            for x in (2 * half, 2 * half + 1):
                for cb in range(4):
                    off = x * 4096 + (16384 if which == "dV" else 0)
                    b = tup((192 if which == "dV" else 208) + 4 * x, 4)
                    reads = [("ds_read_b64_tr_b16 %%s, v%d offset:%d" % (120 + cb, off), 0, 2),
                             ("ds_read_b64_tr_b16 %%s, v%d offset:%d" % (124 + cb, off + 2048), 2, 2)]
                    L.append((which, cb, reads, b, False))
    assert len(L) == 64
    return L


def groups(masked):
    """Vector work as groups: name, earliest slot, deadline slot, lse / delta quad read or None, instructions."""
    G = []
    use = 0
    for qb in range(2):
        s_ready = 12 + 16 * qb           # the S chain ends at slot 7 + 16 qb, the dP chain at 15 + 16 qb
        d_ready = 20 + 16 * qb
        for b4 in range(4):
            ins = []
            if masked:
                for i in range(4):
                    e = 4 * b4 + i
                    c = qb * 32 + 8 * (e >> 2) + (e & 3)
                    ins += [("v_add_u32 v95, %d, %%%d" % (c, OP_TB), 1), ("v_cmp_lt_u32 vcc, v95, %%%d" % OP_LEN, 1),
                            ("v_cndmask_b32 %s, v94, %s, vcc" % (S(qb, e), S(qb, e)), 1)]
            q = use % 4
            for i in range(4):
                ins.append(("v_mul_f32 %s, %s, %s" % (LQ(q, i), NEG_LOG2E, LQ(q, i)), 1))
            for i in range(4):
                ins.append(("v_fma_f32 %s, %s, %%%d, %s" % (S(qb, 4 * b4 + i), S(qb, 4 * b4 + i), OP_SL2, LQ(q, i)), 1))
            for i in range(4):
                ins.append(("v_exp_f32 %s, %s" % (S(qb, 4 * b4 + i), S(qb, 4 * b4 + i)), 2))
            # query chunk x = 2 qb + (b4 >> 1) is consumed by dV at slot 32 + 4 x (x < 2) or 48 + 4 (x - 2)
            x = 2 * qb + (b4 >> 1)
            dl = (32 + 4 * x) if x < 2 else (48 + 4 * (x - 2))
            G.append(dict(name="E%d%d" % (qb, b4), ready=s_ready, deadline=dl, quad=(q, (qb * 32 + 8 * b4) * 4), ins=ins))
            use += 1
            if b4 & 1:
                sl = b4 >> 1
                ins = [("v_cvt_pk_bf16_f32 %s, %s, %s" % (BP(x, j), S(qb, 8 * sl + 2 * j), S(qb, 8 * sl + 2 * j + 1)), 1) for j in range(4)]
                G.append(dict(name="CP%d%d" % (qb, sl), ready=s_ready, deadline=dl, quad=None, ins=ins))
        for b4 in range(4):
            q = use % 4
            ins = []
            for i in range(4):
                e = 4 * b4 + i
                ins.append(("v_sub_f32 %s, %s, %s" % (DP(qb, e), DP(qb, e), LQ(q, i)), 1))
            for i in range(4):
                e = 4 * b4 + i
                ins.append(("v_mul_f32 %s, %s, %s" % (DP(qb, e), S(qb, e), DP(qb, e)), 1))
            x = 2 * qb + (b4 >> 1)
            dl = (40 + 4 * x) if x < 2 else (56 + 4 * (x - 2))
            G.append(dict(name="D%d%d" % (qb, b4), ready=d_ready, deadline=dl, quad=(q, 256 + (qb * 32 + 8 * b4) * 4), ins=ins))
            use += 1
            if b4 & 1:
                sl = b4 >> 1
                ins = [("v_cvt_pk_bf16_f32 %s, %s, %s" % (BS(x, j), DP(qb, 8 * sl + 2 * j), DP(qb, 8 * sl + 2 * j + 1)), 1) for j in range(4)]
                G.append(dict(name="CS%d%d" % (qb, sl), ready=d_ready, deadline=dl, quad=None, ins=ins))
    return G


def schedule(masked, cap):
    """slot -> list of ('valu', text) / ('lq', quad, offset) in issue order.  The list order of the groups is a valid
    program order; earliest deadline first with ties in list order never starts a group before one it depends on,
    because deadlines grow along every dependency chain."""
    G = groups(masked)
    order = {g["name"]: i for i, g in enumerate(G)}
    slots = [[] for _ in range(64)]
    pre = []                                  # before the first MFMA
    # the lse / delta quads rotate over four registers: a quad's read may be issued once the group that used the
    # register before has been issued in full
    quad_users = [g for g in G if g["quad"]]
    done_at = {}
    pending = list(G)
    cur = None
    left = []
    read_issued = set()

    def issue_reads(slot_list, slot):
        for k, g in enumerate(quad_users):
            if g["name"] in read_issued:
                continue
            prev = quad_users[k - 4]["name"] if k >= 4 else None
            if prev is None or (prev in done_at and done_at[prev] <= slot):
                if slot is None or g["ready"] - slot <= 6:      # not far ahead of its use: the in-order LDS queue stays short
                    slot_list.append(("lq", g["quad"][0], g["quad"][1]))
                    read_issued.add(g["name"])

    issue_reads(pre, None)
    for slot in range(64):
        room = cap
        while room > 0:
            if cur is None:
                ready = [g for g in pending if g["ready"] <= slot and (g["quad"] is None or g["name"] in read_issued)]
                if not ready:
                    break
                cur = min(ready, key=lambda g: (g["deadline"], order[g["name"]]))
                pending.remove(cur)
                left = list(cur["ins"])
            text, cost = left[0]
            if cost > room and room < cap:
                break
            slots[slot].append(("valu", text))
            room -= cost
            left.pop(0)
            if not left:
                done_at[cur["name"]] = slot
                assert slot < cur["deadline"], ("deadline missed", cur["name"], slot, cur["deadline"])
                cur = None
        issue_reads(slots[slot], slot)
    assert not pending and cur is None, [g["name"] for g in pending]
    assert len(read_issued) == len(quad_users)
    return pre, slots


def load_ops(k):
    """the k-th load of the tile two steps ahead: Q row groups 0..3, dO row groups 0..3, the lse / delta value"""
    if k == 8:
        return ["s_mov_b32 m0, %%%d" % OP_M0L, "s_nop 0", "global_load_lds_dword %%%d, off" % OP_VL]
    which, i = k // 4, k % 4
    base = "s[80:81]" if which == 0 else "s[82:83]"
    lo, hi = ("s80", "s81") if which == 0 else ("s82", "s83")
    ops = ["s_add_u32 m0, %%%d, %d" % (OP_M0T, which * 16384 + i * 1024),
           "v_xor_b32 v92, %d, %%%d" % (16 * (((i & 1) << 1) | (i >> 1)), OP_VQ if which == 0 else OP_VD),   # the row group's part of the swizzle
           "global_load_lds_dwordx4 v92, %s" % base]
    if i < 3:
        ops += ["s_add_u32 %s, %s, %%%d" % (lo, lo, OP_SQ if which == 0 else OP_SD), "s_addc_u32 %s, %s, 0" % (hi, hi)]
    return ops


def load_prologue():
    return ["s_mov_b32 s86, m0", "s_mov_b64 s[80:81], %%%d" % OP_GQ, "s_mov_b64 s[82:83], %%%d" % OP_GD]


def emit(masked, loads):
    M = mfma_list()
    pre, vslots = schedule(masked, CAP_MASKED if masked else CAP)
    out = []
    lds_issued = 0
    lds_done = 0
    src = {}                                  # register name -> index of the LDS read that fills it
    last_exp = {}                             # register -> instruction index of the v_exp that wrote it
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

    def read(text, key):
        nonlocal lds_issued
        lds_issued += 1
        src[key] = lds_issued
        put(text)

    def frag_reads(m):
        base = 224 + 4 * (m % 8)
        for text, off, n in M[m][2]:
            read(text % tup(base + off, n), "F%d" % (m % 8))

    def do_side(op):
        if op[0] == "lq":
            _, q, off = op
            read("ds_read_b128 %s, %%%d offset:%d" % (tup(96 + 4 * q, 4), OP_AL, off), "LQ%d" % q)
            return
        text = op[1]
        toks = text.replace(",", " ").split()
        regs = [t for t in toks[1:] if t.startswith("v") and t[1:].isdigit()]
        for r in regs:                        # lse / delta quad registers come from LDS
            n = int(r[1:])
            if 96 <= n < 112 and ("LQ%d" % ((n - 96) // 4)) in src:
                wait_lds(src["LQ%d" % ((n - 96) // 4)])
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
        put("v_mov_b32 v94, 0xff800000")
    for ks in range(8):                       # slice addresses: the swizzle is an XOR on the chunk bits, so is the slice
        put("v_xor_b32 v%d, %d, %%%d" % (112 + ks, 32 * ks, OP_AR))
        frag_reads(ks)                        # the first eight MFMAs are the slices of S0
    for cb in range(4):                       # patch addresses: column block cb, rows 0..3 and 8..11 of a query chunk
        put("v_xor_b32 v%d, %d, %%%d" % (120 + cb, 64 * cb, OP_AT))
        put("v_xor_b32 v%d, %d, %%%d" % (124 + cb, (64 * cb) ^ 16, OP_AT))
    for op in pre:
        do_side(op)
    for m in range(64):
        kind = M[m][0]
        wait_lds(src["F%d" % (m % 8)])
        a = F(m % 8)
        if kind in ("S", "dP"):
            qb, b, first = M[m][1], M[m][3], M[m][4]
            d = tup((128 if kind == "S" else 160) + 16 * qb, 16)
            put("v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (d, a, b, "0" if first else d))
        else:
            cb, b = M[m][1], M[m][3]
            d = "%%%d" % ((OP_DV if kind == "dV" else OP_DK) + cb)
            put("v_mfma_f32_32x32x16_bf16 %s, %s, %s, %s" % (d, a, b, d))
        if 8 <= m + 6 < 64:                   # the fragment six slots ahead; its registers were last read by MFMA m - 2
            frag_reads(m + 6)
        if loads and m in LOAD_SLOTS:
            for t in load_ops(LOAD_SLOTS.index(m)):
                put(t)
        for op in vslots[m]:
            do_side(op)
    if loads:
        put("s_mov_b32 m0, s86")
    return out


def loads_only():
    out = load_prologue()
    for k in range(9):
        out += load_ops(k)
    return out + ["s_mov_b32 m0, s86"]


def main(out_path=None):
    lines = []
    # dispatch: %30 = kind (0 none, 1 plain, 2 masked) + 4 * loads
    for mode, body in ((0, []), (1, emit(False, False)), (2, emit(True, False)), (4, loads_only()), (5, emit(False, True)), (6, emit(True, True))):
        lines += ["s_cmp_eq_u32 %%%d, %d" % (OP_MODE, mode), "s_cbranch_scc0 L_dkv_not%d_%%=" % mode] + body + \
                 ["s_branch L_dkv_end_%=", "L_dkv_not%d_%%=:" % mode]
    lines.append("L_dkv_end_%=:")
    out = out_path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "attn_dkv_tile.inc")
    with open(out, "w") as f:
        f.write("// Generated by gen_attn_dkv_tile.py -- do not edit.  One tile step of attn_bwd_dkv3_mfma.\n")
        f.write("#define ATTN_DKV_TILE_ASM \\\n")
        for ln in lines:
            f.write('  "%s\\n" \\\n' % ln)
        f.write('  ""\n')
        vregs = ", ".join('"v%d"' % i for i in range(92, 256))
        f.write("#define ATTN_DKV_TILE_CLOBBERS %s, \"s80\", \"s81\", \"s82\", \"s83\", \"s86\", \"vcc\", \"scc\", \"memory\"\n" % vregs)
    print("wrote", out, len(lines), "instructions")


if __name__ == "__main__":
    import sys
    main(sys.argv[1] if len(sys.argv) > 1 else None)
