"""CPU checks of the generated instruction sequences: the attention backward (csrc/gen_attn_dkv_tile.py,
csrc/gen_attn_dq_tile.py -> attn_dkv_tile.inc, attn_dq_tile.inc), the adapter-gradient loop (lora_grad_loop.inc) and
the projection GEMM's loop (gemm_rs_loop.inc), the last two at the end of the file.

The blocks are hand-placed instruction streams for one wave, so what a compiler would guarantee is checked here by
replaying them:
  * the committed .inc files are what the generators write;
  * every LDS read has been waited for (lgkmcnt, LDS operations complete in order) before its registers are used, is
    not overwritten before the MFMA(s) it was made for, and does not land in the operand of the MFMA issued last;
  * a vector instruction reads a matrix result only four or more MFMAs (or, where the sequence has gaps, forty
    instructions) after the end of its chain (nothing interlocks that read), and reads a v_exp result two or more
    instructions later;
  * every fixed register of a block is on its clobber list;
  * the fragments the MFMAs receive are the ones the mathematics asks for: the LDS image of a tile is built as the
    kernels' loads leave it (16-byte chunk c of row r at position c ^ f(r)), the addresses are the kernels' per-lane
    formulas, ds_read_b64_tr_b16 is replayed with the lane layout found on the device (the 16 lanes of a block each
    supply 4 consecutive elements; lane 4 r + k of the block receives element k of the lanes r, r + 4, r + 8, r + 12),
    and the registers of every MFMA's A operand are compared with the definition of that operand;
  * row reads and patch reads are free of LDS bank conflicts (64 banks of 4 bytes; 16 lanes per pass for 16-byte
    reads, 32 for 8-byte reads)."""
import importlib.util
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_22673_amd", "csrc")


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _macro(path, name):
    text = open(path).read()
    body = text[text.index("#define " + name):]
    lines = []
    for ln in body.splitlines()[1:]:
        m = re.match(r'\s*"(.*)\\n" \\$', ln)
        if not m:
            break
        lines.append(m.group(1))
    return lines


def _clobbers(path, name):
    text = open(path).read()
    line = [l for l in text.splitlines() if l.startswith("#define " + name)][0]
    return set(re.findall(r'"([a-z]+\d*)"', line))


def _bodies(lines, prefix):
    """mode -> instruction list, cut at the dispatch labels"""
    out, cur, mode = {}, None, None
    for ln in lines:
        m = re.match(r"s_cmp_eq_u32 %\d+, (\d+)", ln)
        if m:
            mode, cur = int(m.group(1)), None
            continue
        if ln.startswith("s_cbranch_scc0 L_%s_not" % prefix):
            cur = []
            continue
        if ln.startswith("s_branch L_%s_end" % prefix):
            out[mode] = cur
            cur = None
            continue
        if cur is not None:
            cur.append(ln)
    return out


def _regs(tok):
    """register token -> list of names: v7 -> ['v7'], v[4:7] -> ['v4'..'v7'], %12 -> ['%12'], else []"""
    tok = tok.strip()
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return ["v%d" % i for i in range(int(m.group(1)), int(m.group(2)) + 1)]
    if re.fullmatch(r"v\d+", tok) or re.fullmatch(r"%\d+", tok):
        return [tok]
    return []


def _parse(ln):
    """-> (opcode, written registers, read registers, offset)"""
    op, _, rest = ln.partition(" ")
    off = 0
    m = re.search(r"offset:(\d+)", rest)
    if m:
        off = int(m.group(1))
        rest = rest[:m.start()]
    toks = [t for t in re.split(r",\s*(?![^\[]*\])", rest.strip()) if t]
    if op.startswith("v_mfma"):
        return op, _regs(toks[0]), _regs(toks[1]) + _regs(toks[2]) + _regs(toks[3]), off
    if op.startswith("ds_read"):
        return op, _regs(toks[0]), _regs(toks[1]), off
    if op.startswith("global_load_lds"):
        return op, [], _regs(toks[0]), off
    if op.startswith("v_cmp"):
        return op, [], _regs(toks[1]) + _regs(toks[2]), off
    if op.startswith("v_"):
        reads = []
        for t in toks[1:]:
            reads += _regs(t)
        return op, _regs(toks[0]), reads, off
    return op, [], [], off


def _replay_hazards(ins):
    lds_queue = []                # outstanding LDS reads, oldest first: sets of written registers
    pending = {}                  # register -> True while its LDS read is outstanding
    mfma_count = 0
    mfma_write = {}               # register -> (mfma_count, instruction index) at its last write by an MFMA
    exp_write = {}                # register -> instruction index of the v_exp that wrote it
    frag_owner = {}               # register -> [index of the ds_read that filled it, MFMAs that consumed it]
    frag_regs = set()             # registers that serve as A operands
    mfma_read = {}                # register -> number of MFMAs issued before the last one that read it
    for ln in ins:
        if ln.startswith("v_mfma"):
            frag_regs |= set(_regs([t.strip() for t in re.split(r",\s*(?![^\[]*\])", ln.partition(" ")[2])][1]))
    for idx, ln in enumerate(ins):
        op, wr, rd, _ = _parse(ln)
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", ln)
            if m:
                while len(lds_queue) > int(m.group(1)):
                    for r in lds_queue.pop(0):
                        pending.pop(r, None)
            continue
        for r in rd:
            assert r not in pending, ("register read before its LDS read was waited for", idx, ln, r)
        if op.startswith("v_mfma"):
            for r in rd:
                if r in frag_owner:
                    frag_owner[r][1] += 1
                mfma_read[r] = mfma_count
            mfma_count += 1
            for r in wr:
                mfma_write[r] = (mfma_count, idx)
                exp_write.pop(r, None)
            continue
        if op.startswith("ds_read"):
            for r in wr:
                assert r not in pending, ("LDS read into a register with a read outstanding", idx, ln)
                # the MFMA that read the register last has another one behind it: it has taken its operands
                assert r not in mfma_read or mfma_count - mfma_read[r] >= 2, ("LDS read into the operand of the MFMA just issued", idx, ln)
                if r in frag_owner and r in frag_regs:
                    assert frag_owner[r][1] > 0, ("fragment overwritten before any MFMA used it", idx, ln, r)
                frag_owner[r] = [idx, 0]
                pending[r] = True
                mfma_write.pop(r, None)
            lds_queue.append(list(wr))
            while len(lds_queue) > 15:        # the counter has four bits: the wave does not issue another LDS operation before the oldest is back
                for r in lds_queue.pop(0):
                    pending.pop(r, None)
            continue
        if op.startswith("v_") or op.startswith("global_load_lds"):
            for r in rd:
                if r in mfma_write:
                    assert mfma_count - mfma_write[r][0] >= 4 or idx - mfma_write[r][1] >= 40, ("matrix result read too early", idx, ln, r)
                if r in exp_write and not op.startswith("v_exp"):
                    assert idx - exp_write[r] >= 2, ("v_exp result read by the next instruction", idx, ln, r)
            for r in wr:
                mfma_write.pop(r, None)
                exp_write.pop(r, None)
                if op.startswith("v_exp"):
                    exp_write[r] = idx
    assert not lds_queue, "LDS reads still outstanding at the end of the block"
    assert all(v[1] > 0 for r, v in frag_owner.items() if r in frag_regs), "a fragment was read from LDS and never used"
    return mfma_count


def _fixed_registers(ins):
    out = set()
    for ln in ins:
        _, wr, rd, _ = _parse(ln)
        out |= {r for r in wr + rd if r.startswith("v")}
        out |= {"s" + x for x in re.findall(r"\bs(\d+)\b", ln)}
        for a, b in re.findall(r"s\[(\d+):(\d+)\]", ln):
            out |= {"s%d" % i for i in range(int(a), int(b) + 1)}
    return out


CASES = [("gen_attn_dkv_tile", "attn_dkv_tile.inc", "ATTN_DKV_TILE", "dkv", 64), ("gen_attn_dq_tile", "attn_dq_tile.inc", "ATTN_DQ_TILE", "dq", 96)]


@pytest.mark.parametrize("gen,inc,macro,prefix,n_mfma", CASES)
def test_committed_file_is_what_the_generator_writes(gen, inc, macro, prefix, n_mfma, tmp_path):
    mod = _load(gen)
    out = tmp_path / inc
    mod.main(str(out))
    assert open(out).read() == open(os.path.join(CSRC, inc)).read()


@pytest.mark.parametrize("gen,inc,macro,prefix,n_mfma", CASES)
def test_waits_hazards_and_clobbers(gen, inc, macro, prefix, n_mfma):
    path = os.path.join(CSRC, inc)
    bodies = _bodies(_macro(path, macro + "_ASM"), prefix)
    clob = _clobbers(path, macro + "_CLOBBERS")
    assert {m & 3 for m in bodies} >= {1, 2}
    for mode, ins in bodies.items():
        n = _replay_hazards(ins)
        assert n == (n_mfma if mode & 3 else 0), (mode, n)
        assert _fixed_registers(ins) <= clob, (mode, sorted(_fixed_registers(ins) - clob)[:8])
        loads = sum(1 for ln in ins if ln.startswith("global_load_lds"))
        assert loads == ((9 if prefix == "dkv" else 8) if mode & 4 else 0), (mode, loads)


# ---------------------------------------------------------------- what the MFMAs receive

def _f(row):
    return ((row & 3) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1)


def _lds_image(n_tiles):
    """tiles of [64][128] elements, element id = tile * 8192 + row * 128 + column, stored as the kernels' loads store them"""
    img = np.zeros(n_tiles * 8192, dtype=np.int64)
    for t in range(n_tiles):
        for row in range(64):
            for c in range(16):
                g = c ^ _f(row & 15)
                img[t * 8192 + row * 128 + c * 8: t * 8192 + row * 128 + c * 8 + 8] = t * 8192 + row * 128 + g * 8 + np.arange(8)
    return img


def _lane_addresses():
    aR, aT = np.zeros(64, dtype=np.int64), np.zeros(64, dtype=np.int64)
    for lane in range(64):
        l31, h, sl, mh = lane & 31, lane >> 5, lane & 15, (lane >> 4) & 1
        row0 = 4 * h + (sl >> 2)
        aR[lane] = l31 * 256 + ((h ^ _f(l31 & 15)) * 16)
        aT[lane] = row0 * 256 + (((2 * mh + ((sl & 3) >> 1)) ^ _f(row0)) * 16) + (sl & 1) * 8
    return aR, aT


def _bank_conflicts(addr, nbytes, group):
    worst = 1
    for g0 in range(0, 64, group):
        banks = {}
        for lane in range(g0, g0 + group):
            for w in range(int(addr[lane]) // 4, (int(addr[lane]) + nbytes) // 4):
                banks.setdefault(w % 64, set()).add(w)
        worst = max(worst, max(len(v) for v in banks.values()))
    return worst


def _replay_fragments(ins, op_ar, op_at, n_tiles):
    """-> per MFMA: (destination token, B token, A fragment as [64 lanes][8] element ids); checks the banks on the way"""
    img = _lds_image(n_tiles)
    aR, aT = _lane_addresses()
    vreg = {"%%%d" % op_ar: aR, "%%%d" % op_at: aT}
    out = []
    for ln in ins:
        op, wr, rd, off = _parse(ln)
        if op == "v_xor_b32":
            toks = [t.strip() for t in ln.partition(" ")[2].split(",")]
            if toks[2] in vreg:
                vreg[toks[0]] = vreg[toks[2]] ^ int(toks[1])
        elif op == "ds_read_b128" and rd[0] in vreg and int(wr[0][1:]) >= 64:
            a = vreg[rd[0]] + off
            assert _bank_conflicts(a, 16, 16) == 1, ln
            val = np.stack([img[a // 2 + j] for j in range(8)], axis=1)
            for k in range(4):
                vreg[wr[k]] = val[:, 2 * k:2 * k + 2]
        elif op == "ds_read_b64_tr_b16":
            a = vreg[rd[0]] + off
            assert _bank_conflicts(a, 8, 32) == 1, ln
            val = np.zeros((64, 4), dtype=np.int64)
            for blk in range(4):
                for L in range(16):
                    k, r = L % 4, L // 4
                    for j in range(4):
                        val[blk * 16 + L, j] = img[a[blk * 16 + 4 * j + r] // 2 + k]
            vreg[wr[0]], vreg[wr[1]] = val[:, 0:2], val[:, 2:4]
        elif op.startswith("v_mfma"):
            toks = [t.strip() for t in re.split(r",\s*(?![^\[]*\])", ln.partition(" ")[2])]
            a_regs = _regs(toks[1])
            out.append((toks[0], toks[2], np.concatenate([vreg[r] for r in a_regs], axis=1)))
    return out


def _expect_rows(tile, rb):
    """A operand [32 rows of the tile block rb] x [16 of head_dim]: lane (l31, h) holds row l31, columns 8 h .. 8 h + 7 of the slice"""
    def want(lane, j, ks):
        return tile * 8192 + (rb * 32 + (lane & 31)) * 128 + ks * 16 + (lane >> 5) * 8 + j
    return want


def _expect_cols(tile, cb, x):
    """A operand [32 columns of block cb] x [16 rows of chunk x], rows in the order the B operand holds them"""
    def want(lane, j):
        row = 16 * x + 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3)
        return tile * 8192 + row * 128 + cb * 32 + (lane & 31)
    return want


def test_dkv_fragments():
    g = _load("gen_attn_dkv_tile")
    ins = _bodies(_macro(os.path.join(CSRC, "attn_dkv_tile.inc"), "ATTN_DKV_TILE_ASM"), "dkv")[1]
    frs = _replay_fragments(ins, g.OP_AR, g.OP_AT, 2)                  # tile 0 = Q, tile 1 = dO
    assert len(frs) == 64
    seen = set()
    for dst, b, a in frs:
        lanes, js = np.arange(64)[:, None], np.arange(8)[None, :]
        if dst.startswith("v["):                                        # S or dP of query block qb, slice from the B operand
            base = int(re.match(r"v\[(\d+):", dst).group(1))
            kind, qb = ("S", (base - 128) // 16) if base < 160 else ("dP", (base - 160) // 16)
            ks = int(b[1:]) - (g.OP_KF if kind == "S" else g.OP_VF)
            want = _expect_rows(0 if kind == "S" else 1, qb)(lanes, js, ks)
            seen.add((kind, qb, ks))
        else:                                                           # dV / dK column block, query chunk from the B operand
            o = int(dst[1:])
            kind, cb = ("dK", o - g.OP_DK) if o < g.OP_DV else ("dV", o - g.OP_DV)
            bbase = int(re.match(r"v\[(\d+):", b).group(1))
            x = (bbase - (192 if kind == "dV" else 208)) // 4
            assert (kind == "dV") == (bbase < 208)
            want = _expect_cols(1 if kind == "dV" else 0, cb, x)(lanes, js)
            seen.add((kind, cb, x))
        assert np.array_equal(a, want), (dst, b)
    assert len(seen) == 64


def test_dq_fragments():
    g = _load("gen_attn_dq_tile")
    ins = _bodies(_macro(os.path.join(CSRC, "attn_dq_tile.inc"), "ATTN_DQ_TILE_ASM"), "dq")[1]
    frs = _replay_fragments(ins, g.OP_AR, g.OP_AT, 2)                  # tile 0 = K, tile 1 = V
    assert len(frs) == 96
    seen = set()
    lanes, js = np.arange(64)[:, None], np.arange(8)[None, :]
    for dst, b, a in frs:
        if dst.startswith("v["):
            base = int(re.match(r"v\[(\d+):", dst).group(1))
            kind, t = ("S", (base - 128) // 16) if base < 192 else ("dP", (base - 192) // 16)
            qb, kb = t >> 1, t & 1
            o = int(b[1:]) - (g.OP_QF if kind == "S" else g.OP_DOF)
            assert o // 8 == qb
            want = _expect_rows(0 if kind == "S" else 1, kb)(lanes, js, o % 8)
            seen.add((kind, qb, kb, o % 8))
        else:
            o = int(dst[1:]) - g.OP_DQ
            qb, cb = o // 4, o % 4
            bbase = int(re.match(r"v\[(\d+):", b).group(1))
            assert (bbase - 96) // 16 == qb
            x = ((bbase - 96) % 16) // 4
            want = _expect_cols(0, cb, x)(lanes, js)
            seen.add(("dQ", qb, cb, x))
        assert np.array_equal(a, want), (dst, b)
    assert len(seen) == 96


def test_the_load_swizzle_of_a_row_group_is_the_xor_the_blocks_use():
    """A load instruction of a wave fills four rows; lane -> row lane / 16 of the group, position lane % 16.  The blocks
    take the lane's offset of row group 0 and XOR a constant per group: that must be the chunk c ^ f(row)."""
    for gen in ("gen_attn_dkv_tile", "gen_attn_dq_tile"):
        g = _load(gen)
        for i in range(4):
            text = [t for t in g.load_ops(i) if t.startswith("v_xor_b32")][0]
            const = int(text.split(",")[1])
            for wave in range(4):
                for lane in range(64):
                    l4, c = lane >> 4, lane & 15
                    row = wave * 16 + 4 * i + l4
                    assert ((c ^ _f(l4)) * 16) ^ const == (c ^ _f(row & 15)) * 16


def _min_valu_to_mfma_distance(ins):
    last, best = {}, 10 ** 6
    for idx, ln in enumerate(ins):
        op, wr, rd, _ = _parse(ln)
        if op.startswith("v_mfma"):
            for r in rd:
                if r in last:
                    best = min(best, idx - last[r])
        elif op.startswith("v_"):
            for r in wr:
                last[r] = idx
    return best


@pytest.mark.parametrize("gen,inc,macro,prefix,n_mfma", CASES)
def test_an_mfma_never_reads_a_register_a_vector_instruction_just_wrote(gen, inc, macro, prefix, n_mfma):
    """Operands built by vector instructions directly in front of the MFMA that reads them gave wrong results in the
    adapter-gradient loop (with two temporaries in turn); every block keeps a distance."""
    bodies = _bodies(_macro(os.path.join(CSRC, inc), macro + "_ASM"), prefix)
    for mode, ins in bodies.items():
        assert _min_valu_to_mfma_distance(ins) >= 8, mode


# ---------------------------------------------------------------- the adapter-gradient loop

def test_lora_grad_loop():
    """lora_grad_loop.inc: current; loads are waited for before use (vmcnt, loads return in order) and never land in
    registers that instructions issued less than a step ago still read; operands are built a column ahead."""
    mod = _load("gen_lora_grad_loop")
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "lora_grad_loop.inc")
        mod.main(out)
        assert open(out).read() == open(os.path.join(CSRC, "lora_grad_loop.inc")).read()
    lines = _macro(os.path.join(CSRC, "lora_grad_loop.inc"), "LORA_GRAD_LOOP_ASM")
    clob = _clobbers(os.path.join(CSRC, "lora_grad_loop.inc"), "LORA_GRAD_LOOP_CLOBBERS")
    assert _fixed_registers(lines) <= clob
    start = lines.index("L_tn_loop_%=:")
    end = lines.index("L_tn_end_%=:")
    body = [ln for ln in lines[start + 1:end] if not ln.startswith("s_cbranch")]
    seq = lines[:start] + body + body + body                   # three trips: the steady state
    queue, pending, last_read = [], {}, {}
    n_mfma = 0
    for idx, ln in enumerate(seq):
        op, wr, rd, _ = _parse(ln)
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", ln)
            if m:
                while len(queue) > int(m.group(1)):
                    for r in queue.pop(0):
                        pending.pop(r, None)
            continue
        if op.startswith("global_load_dwordx4"):
            toks = [t.strip() for t in re.split(r",\s*(?![^\[]*\])", ln.partition(" ")[2])]
            dst = _regs(toks[0])
            for r in dst:
                assert r not in pending
                assert idx - last_read.get(r, -10 ** 6) > 16, ("load issued right behind a read of its register", idx, ln)
                pending[r] = True
            queue.append(dst)
            assert len(queue) < 64
            continue
        for r in rd:
            assert r not in pending, ("register used before its load was waited for", idx, ln, r)
            last_read[r] = idx
        n_mfma += op.startswith("v_mfma")
    assert n_mfma == 3 * 4 * 32
    assert _min_valu_to_mfma_distance(seq) >= 4


# ---------------------------------------------------------------- the projection GEMM's loop

def _replay_gemm_loop(lines):
    """the loop replayed over the prologue and three trips of the two-step loop body, with counters kept
    independently of the generator's own: a register is not used while a global load or an LDS read into it is
    outstanding (vmcnt / lgkmcnt, both complete in order); a global load does not land in registers whose LDS store
    may still be reading them; every MFMA's fragments come from the LDS stage and slice its step is on; a step's
    fragment reads never touch an LDS stage that stores issued since the last barrier are writing."""
    start, end = lines.index("L_rs_loop_%=:"), lines.index("L_rs_end_%=:")
    body = [ln for ln in lines[start + 1:end] if not ln.startswith("s_cbranch")]
    seq = lines[:start] + body * 3
    vm_q, lds_q = [], []                      # outstanding global loads / LDS operations, oldest first
    vm_pending, lds_pending = {}, {}          # register -> True while a load / an LDS read into it is outstanding
    store_reads = {}                          # register -> True while an LDS store that reads it is outstanding
    written_since_barrier, read_since_barrier = set(), set()     # LDS stages (0/1 for A, 2/3 for B)
    n_mfma = 0

    def stage_of(addr_reg, off):
        # A stages at LDS offsets 0 / 32768, B stages at 65536 / 98304 (the B part sits in the address registers)
        a = int(addr_reg[1:])
        is_b = a in (196, 197, 198, 199, 202, 203)
        return (2 if is_b else 0) + (off // 32768)

    for idx, ln in enumerate(seq):
        op = ln.split()[0]
        toks = [t.strip() for t in re.split(r",\s*(?![^\[]*\])", ln.partition(" ")[2])]
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", ln)
            if m:
                while len(vm_q) > int(m.group(1)):
                    for r in vm_q.pop(0):
                        vm_pending.pop(r, None)
            m = re.search(r"lgkmcnt\((\d+)\)", ln)
            if m:
                while len(lds_q) > int(m.group(1)):
                    kind, regs = lds_q.pop(0)
                    for r in regs:
                        (lds_pending if kind == "read" else store_reads).pop(r, None)
            continue
        if op == "s_barrier":
            assert not lds_q, ("LDS operations outstanding at the barrier", idx)
            written_since_barrier, read_since_barrier = set(), set()
            continue
        if op == "global_load_dwordx4":
            dst = _regs(toks[0])
            for r in dst:
                assert r not in vm_pending and r not in store_reads, ("load into registers still in use", idx, ln)
                vm_pending[r] = True
            vm_q.append(dst)
            assert len(vm_q) <= 63
            continue
        if op == "ds_write_b128":
            off = int(re.search(r"offset:(\d+)", ln).group(1)) if "offset:" in ln else 0
            src = _regs(toks[1].split(" offset")[0])
            for r in src:
                assert r not in vm_pending, ("LDS store of a register whose load was not waited for", idx, ln)
                store_reads[r] = True
            st = stage_of(toks[0], off)
            assert st not in read_since_barrier, ("store into an LDS stage that is being read", idx, ln)
            written_since_barrier.add(st)
            lds_q.append(("write", src))
            while len(lds_q) > 15:
                kind, regs = lds_q.pop(0)
                for r in regs:
                    (lds_pending if kind == "read" else store_reads).pop(r, None)
            continue
        if op == "ds_read_b128":
            off = int(re.search(r"offset:(\d+)", ln).group(1)) if "offset:" in ln else 0
            dst = _regs(toks[0])
            addr = toks[1].split(" offset")[0].strip()
            if addr.startswith("v"):
                st = stage_of(addr, off)
                assert st not in written_since_barrier, ("fragment read from an LDS stage written since the barrier", idx, ln)
                read_since_barrier.add(st)
            for r in dst:
                assert r not in lds_pending
                lds_pending[r] = True
            lds_q.append(("read", dst))
            while len(lds_q) > 15:
                kind, regs = lds_q.pop(0)
                for r in regs:
                    (lds_pending if kind == "read" else store_reads).pop(r, None)
            continue
        if op.startswith("v_mfma"):
            for r in _regs(toks[1]) + _regs(toks[2]):
                assert r not in lds_pending and r not in vm_pending, ("MFMA on a fragment that was not waited for", idx, ln)
            n_mfma += 1
            continue
        if op.startswith("v_"):
            for t in toks[1:]:
                for r in _regs(t):
                    assert r not in lds_pending and r not in vm_pending, (idx, ln)
    return n_mfma


def test_gemm_rs_loop_replay():
    lines = _macro(os.path.join(CSRC, "gemm_rs_loop.inc"), "GEMM_RS_LOOP_ASM")
    assert _replay_gemm_loop(lines) == 3 * 2 * 64
    # the replay has teeth: planted mistakes inside the loop body are caught
    loop_at = lines.index("L_rs_loop_%=:")

    def without(pred, count=1):
        out, left = [], count
        for i, ln in enumerate(lines):
            if left and i > loop_at and pred(ln):
                left -= 1
                continue
            out.append(ln)
        assert left == 0
        return out

    for planted in (without(lambda ln: ln.startswith("s_waitcnt vmcnt")),             # a store of data that has not arrived
                    without(lambda ln: ln.startswith("s_waitcnt lgkmcnt("), 3),      # an MFMA on fragments still on their way
                    without(lambda ln: ln == "s_barrier")):                          # a stage rewritten while it is read
        with pytest.raises(AssertionError):
            _replay_gemm_loop(planted)
