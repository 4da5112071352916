#!/usr/bin/env python3
"""Writes lora_grad_loop.inc: the streaming loop of lora_grad_tn_kernel (lora_grad.hip, four 16-column blocks of the
narrow operand) as one inline-asm block.  Run by hand after a change (python gen_lora_grad_loop.py); the generated file
is committed.

The kernel is a single pass over a big activation at memory speed, one workgroup per CU (the 128 accumulator registers
of a wave live in the accumulation half of the register file), so what a wave keeps in flight is all its SIMD asks of
memory.  A step is 32 tokens: per lane eight 16-byte loads of the big operand (an 8-token x 8-column block) and four of
the narrow one, 32 v_perm_b32 that transpose the block in registers, 32 v_mfma_f32_16x16x32_bf16.  The loop keeps FOUR
register sets: three steps are in flight while one is multiplied (96 KB per CU; 6 TB/s over 256 CUs at 1.5 us of
latency needs 36 KB, and the compiler-built loop with two sets had 32).  Loads return in order, so the wait before a
step's first use is vmcnt(24): the 24 loads of the two younger steps.  Loads past the last step re-read the last step
(the address stops advancing), which keeps that count uniform.

Operands: %0..%31 accumulators (column of the block q, 16-column block nb) -> %(4 q + nb); %32..%39 this lane's byte
offsets of the eight token rows of a block in the big operand; %40..%43 its byte offsets in the four row groups of the
token-major narrow operand; %44, %45 addresses of the first step's block row of both operands (scalar pairs); %46 bytes
between steps in the big operand; %47 number of steps (> 0).
Fixed registers (clobbered): v[52:63] three A operands in rotation, v[64:255] four sets of 48 (eight 4-register loads of the big
operand, four of the narrow one); s[80:83] running addresses, s84 steps done, s85 the step whose loads are issued next,
s86, s87 address increments, s88, s89 the two byte selectors of the transposition.
"""
import os

OP_VX, OP_VU, OP_GX, OP_GU, OP_STR, OP_N = 32, 40, 44, 45, 46, 47
NSET = 4


def X(s, r): return "v[%d:%d]" % (64 + 48 * s + 4 * r, 64 + 48 * s + 4 * r + 3)
def Xd(s, r, c): return "v%d" % (64 + 48 * s + 4 * r + c)
def U(s, nb): return "v[%d:%d]" % (64 + 48 * s + 32 + 4 * nb, 64 + 48 * s + 32 + 4 * nb + 3)
def A(i): return "v[%d:%d]" % (52 + 4 * i, 52 + 4 * i + 3)
def Ad(i, d): return "v%d" % (52 + 4 * i + d)


def loads(s):
    """the twelve loads of the step s85 into set s, then the advance of the addresses (none past the last step)"""
    L = [["global_load_dwordx4 %s, %%%d, s[80:81]" % (X(s, r), OP_VX + r)] for r in range(8)]
    L += [["global_load_dwordx4 %s, %%%d, s[82:83]" % (U(s, nb), OP_VU + nb)] for nb in range(4)]
    adv = ["s_add_u32 s85, s85, 1", "s_cmp_lt_u32 s85, %%%d" % OP_N, "s_cselect_b32 s86, %%%d, 0" % OP_STR, "s_cselect_b32 s87, 64, 0",
           "s_add_u32 s80, s80, s86", "s_addc_u32 s81, s81, 0", "s_add_u32 s82, s82, s87", "s_addc_u32 s83, s83, 0"]
    return L, adv


def body(k):
    """step in set k: wait for it, multiply, and behind the MFMAs issue the loads of the step three ahead into set k + 3"""
    out = ["s_waitcnt vmcnt(24)"]
    L, adv = loads((k + 3) % NSET)
    pending = [x for l in L for x in l]
    n = 0

    def perms(q):                             # column q of the 8 x 8 block as an A operand: dword d = (row 2 d, row 2 d + 1)
        return ["v_perm_b32 %s, %s, %s, %s" % (Ad(q % 3, d), Xd(k, 2 * d + 1, q >> 1), Xd(k, 2 * d, q >> 1), "s89" if q & 1 else "s88") for d in range(4)]

    out += perms(0)
    for q in range(8):
        if q < 7:                             # the operand of the next column is built under this column's MFMAs, into the third
            out += perms(q + 1)               # temporary: with the v_perm directly in front of its MFMAs and two temporaries the results were wrong
        for nb in range(4):
            out.append("v_mfma_f32_16x16x32_bf16 %%%d, %s, %s, %%%d" % (4 * q + nb, A(q % 3), U(k, nb), 4 * q + nb))
            n += 1
            # the loads may only overwrite set k + 3 = k - 1, whose last readers were issued a step ago; twelve loads behind 32 MFMAs
            if n in (2, 4, 7, 9, 12, 14, 17, 19, 22, 24, 27, 29):
                out.append(pending.pop(0))
    assert not pending
    return out + adv


def main(out_path=None):
    e = ["s_mov_b64 s[80:81], %%%d" % OP_GX, "s_mov_b64 s[82:83], %%%d" % OP_GU, "s_mov_b32 s84, 0", "s_mov_b32 s85, 0",
         "s_mov_b32 s88, 0x05040100", "s_mov_b32 s89, 0x07060302"]
    for s in range(3):                        # steps 0, 1, 2 (or the last step again, when there are fewer)
        L, adv = loads(s)
        e += [x for l in L for x in l] + adv
    e.append("L_tn_loop_%=:")
    for k in range(NSET):
        e += body(k)
        e += ["s_add_u32 s84, s84, 1", "s_cmp_ge_u32 s84, %%%d" % OP_N]
        e.append("s_cbranch_scc1 L_tn_end_%=" if k < NSET - 1 else "s_cbranch_scc0 L_tn_loop_%=")
    e += ["L_tn_end_%=:", "s_waitcnt vmcnt(0)", "s_nop 15", "s_nop 15"]
    out = out_path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "lora_grad_loop.inc")
    with open(out, "w") as f:
        f.write("// Generated by gen_lora_grad_loop.py -- do not edit.  Streaming loop of lora_grad_tn_kernel.\n")
        f.write("#define LORA_GRAD_LOOP_ASM \\\n")
        for ln in e:
            f.write('  "%s\\n" \\\n' % ln)
        f.write('  ""\n')
        vregs = ", ".join('"v%d"' % i for i in range(52, 256))
        sregs = ", ".join('"s%d"' % i for i in range(80, 90))
        f.write("#define LORA_GRAD_LOOP_CLOBBERS %s, %s, \"scc\", \"memory\"\n" % (vregs, sregs))
    print("wrote", out, len(e), "instructions")


if __name__ == "__main__":
    import sys
    main(sys.argv[1] if len(sys.argv) > 1 else None)
