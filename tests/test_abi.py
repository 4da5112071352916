"""The C interface without a GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2503_22673_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "actionstudio.h")).read()
    declared = set(re.findall(r"\b(as_[a-z0-9_]+)\s*\(", header))
    declared -= {"as_status"}
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_config_validation(B):
    sh = synth.CONFIGS[1]
    ok = B.make_config(sh)
    ctx = B.Context(ok)
    ctx.close()
    bad = [dict(head_dim=48), dict(n_q_heads=3), dict(struct_size=4), dict(lora_rank=0), dict(lora_targets=0),
           dict(mode=7), dict(n_experts=8, top_k=1), dict(n_experts=6, top_k=2), dict(n_experts=8, top_k=2, lora_targets=0x1f),
           dict(lora_targets=0x81), dict(n_experts=8, top_k=2, train_mode=1, lora_rank=0, lora_targets=0), dict(recompute=5), dict(vocab=1), dict(lora_rank=1000)]
    for kw in bad:
        c = B.make_config(sh)
        for k, v in kw.items():
            setattr(c, k, v)
        with pytest.raises(B.ASError) as e:
            B.Context(c)
        assert e.value.code == B.ERR["CONFIG"], kw
    moe = B.make_config(synth.CONFIGS[5])
    B.Context(moe).close()
    h = C.c_void_p()
    assert B.lib.as_create(C.byref(h), None, 0) == B.ERR["NULL"]
    assert b"NULL" in B.lib.as_last_error(None)


def test_workspace_query(B):
    ctx = B.Context(B.make_config(synth.CONFIGS[1]))
    small = ctx.workspace_bytes(1, 512)
    big = ctx.workspace_bytes(4, 512)
    assert 0 < small < big and small % 256 == 0
    with pytest.raises(B.ASError) as e:
        ctx.workspace_bytes(0, 512)
    assert e.value.code == B.ERR["SHAPE"]
    # config 3 with recompute must fit one MI355X (288 GB) with room for weights
    c3 = B.Context(B.make_config(synth.CONFIGS[3]))
    gb = c3.workspace_bytes(4, 16384) / 2 ** 30
    assert gb < 240, gb            # + 16 GB of bf16 weights + adapters and their moments < 288 GB
    # config 5 (sparse layers, 2 x 8192 tokens): + 93 GB of bf16 weights
    c5 = B.Context(B.make_config(synth.CONFIGS[5]))
    gb5 = c5.workspace_bytes(2, 8192) / 2 ** 30
    assert gb5 < 170, gb5


def _pack_args(trajs):
    return synth.flatten_trajectories(trajs)


def test_pack_rejects_bad_input_on_the_host(B):
    """None of these reaches a HIP call, so they run without a GPU."""
    ctx = B.Context(B.make_config(synth.CONFIGS[1]))
    U, A = 1, 2
    good = [[(U, np.array([1, 2, 3])), (A, np.array([4, 5]))]]
    cases = [
        ([[(7, np.array([1]))]], dict(), "ROLE"),
        ([[(U, np.array([5000]))]], dict(), "TOKEN_RANGE"),
        ([[(U, np.array([-1]))]], dict(), "TOKEN_RANGE"),
        ([[(U, np.arange(20))]], dict(row_len=8, truncate=False), "TOO_LONG"),
        (good, dict(row_len=0), "SHAPE"),
        (good, dict(max_rows=-1), "SHAPE"),
    ]
    for trajs, kw, code in cases:
        tt, to, tr, jo = _pack_args(trajs)
        with pytest.raises(B.ASError) as e:
            ctx.pack(tt, to, tr, jo, kw.get("row_len", 16), kw.get("max_rows", 2), truncate=kw.get("truncate", True),
                     outputs=(None, None, None))
        assert e.value.code in (B.ERR[code], B.ERR["NULL"]), (code, str(e.value))
    # with dummy non-NULL outputs the specific code must come back
    class Fake:
        is_cuda = False
        def data_ptr(self):
            return 4096
    for trajs, kw, code in cases:
        tt, to, tr, jo = _pack_args(trajs)
        with pytest.raises(B.ASError) as e:
            ctx.pack(tt, to, tr, jo, kw.get("row_len", 16), kw.get("max_rows", 2), truncate=kw.get("truncate", True),
                     outputs=(Fake(), Fake(), Fake()))
        assert e.value.code == B.ERR[code], (code, str(e.value))
    tt, to, tr, jo = _pack_args(good)
    bad_off = to.copy(); bad_off[1] = 9; bad_off[2] = 3
    with pytest.raises(B.ASError) as e:
        ctx.pack(tt, bad_off, tr, jo, 16, 2, outputs=(Fake(), Fake(), Fake()))
    assert e.value.code == B.ERR["SHAPE"]


def test_train_step_rejects_bad_segment_tables_on_the_host(B):
    sh = synth.CONFIGS[1]
    ctx = B.Context(B.make_config(sh))
    L = sh.n_layers
    lw = (B.LayerWeights * L)()
    for l in range(L):
        for f, _ in B.LayerWeights._fields_:
            setattr(lw[l], f, 4096)
    W = B.Weights(4096, 4096, 4096, lw)
    ll, lg = (B.LayerLora * L)(), (B.LayerLora * L)()
    for l in range(L):
        for i in range(4):
            ll[l].a[i] = ll[l].b[i] = lg[l].a[i] = lg[l].b[i] = 4096
    lora, grads = B.Lora(ll), B.Grads()
    grads.lora_layers = lg
    p = C.c_void_p(4096)

    def call(cu, n_rows=1, row_len=512, ws=p, ws_bytes=1 << 40, lora_=lora):
        cu = np.asarray(cu, dtype=np.int32)
        return B.lib.as_train_step(ctx.handle, C.byref(W), C.byref(lora_) if lora_ is not None else None, p, p,
                                   cu.ctypes.data_as(C.c_void_p), len(cu) - 1, None, p, n_rows, row_len, p, p, p,
                                   C.byref(grads), ws, ws_bytes, None)

    E = B.ERR
    assert call([1, 512]) == E["CU_SEQLENS"]                       # does not start at 0
    assert call([0, 100, 100, 512]) == E["CU_SEQLENS"]             # not strictly increasing
    assert call([0, 100, 500]) == E["CU_SEQLENS"]                  # does not end at N
    assert call([0, 300, 700, 1024], n_rows=2) == E["CU_SEQLENS"]  # crosses a row end
    assert b"row end" in B.lib.as_last_error(ctx.handle)
    assert call([0, 512], ws=None) == E["WORKSPACE"]
    assert call([0, 512], ws=C.c_void_p(4097)) == E["WORKSPACE"]   # misaligned
    assert call([0, 512], ws_bytes=1024) == E["WORKSPACE"]         # too small
    assert call([0, 512], lora_=None) == E["NULL"]
    assert call([0, 512], n_rows=0) == E["SHAPE"]
    ll[1].b[2] = None
    assert call([0, 512]) == E["NULL"]
    assert b"target v in layer 1" in B.lib.as_last_error(ctx.handle)


def test_adamw_and_op_argument_checks(B):
    ctx = B.Context(B.make_config(synth.CONFIGS[1]))
    one = (C.c_void_p * 1)(4096)
    numel = (C.c_int64 * 1)(16)
    wd = (C.c_uint8 * 1)(1)
    f = B.lib.as_adamw_update
    assert f(ctx.handle, one, None, one, one, one, numel, wd, 1, 0, 1e-3, 0.9, 0.95, 1e-8, 0.0, None) == B.ERR["SHAPE"]
    assert f(ctx.handle, one, None, one, one, one, numel, wd, 1, 1, 1e-3, 1.0, 0.95, 1e-8, 0.0, None) == B.ERR["SHAPE"]
    assert f(ctx.handle, None, None, one, one, one, numel, wd, 1, 1, 1e-3, 0.9, 0.95, 1e-8, 0.0, None) == B.ERR["NULL"]
    nul = (C.c_void_p * 1)(None)
    assert f(ctx.handle, one, None, nul, one, one, numel, wd, 1, 1, 1e-3, 0.9, 0.95, 1e-8, 0.0, None) == B.ERR["NULL"]
    g = B.lib.as_op_gemm
    p = C.c_void_p(4096)
    assert g(ctx.handle, 0, 0, 4, 4, None, 4, p, 4, 4, None, 0, None, 0, 0, 1.0, None, 0, p, 4, 0, None, 0, None) == B.ERR["NULL"]
    assert g(ctx.handle, 0, 0, 4, 4, p, 2, p, 4, 4, None, 0, None, 0, 0, 1.0, None, 0, p, 4, 0, None, 0, None) == B.ERR["SHAPE"]
    assert g(ctx.handle, 9, 0, 4, 4, p, 4, p, 4, 4, None, 0, None, 0, 0, 1.0, None, 0, p, 4, 0, None, 0, None) == B.ERR["CONFIG"]


def test_generated_gemm_loop_is_the_generators_output(tmp_path):
    """The committed inline-asm loop of the register-staged GEMM is what its generator writes (the generator also
    checks, while replaying the instruction sequence, that every wait count fits its counter)."""
    import subprocess, sys
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2503_22673_amd", "csrc")
    out = tmp_path / "loop.inc"
    subprocess.run([sys.executable, os.path.join(csrc, "gen_gemm_rs_loop.py"), str(out)], check=True, capture_output=True)
    assert out.read_text() == open(os.path.join(csrc, "gemm_rs_loop.inc")).read()


def test_row_counted_gemm_and_timing_filter_reject_bad_arguments(B):
    """Host-side checks only: none of these reaches a HIP call."""
    ctx = B.Context(B.make_config(synth.CONFIGS[1]))
    p = C.c_void_p(4096)
    def rows(A=p, Bm=p, Cm=p, M=512, N=256, K=64, lda=64, ldb=64, ldc=256, d_rows=p, row_off=0, d_grp=None, group=0, n_groups=0, stride=0, cap=0):
        return B.lib.as_op_gemm_rows(ctx.handle, B.AS_BF16, 0, M, N, A, lda, Bm, ldb, K, 1.0, None, 0, Cm, ldc, 0,
                                     d_rows, row_off, d_grp, group, n_groups, stride, cap, None)
    assert rows(A=None) == B.ERR["NULL"]
    assert rows(d_rows=None) == B.ERR["NULL"]                              # neither a row count nor a group table
    assert rows(M=-1) == B.ERR["SHAPE"] and rows(row_off=-1) == B.ERR["SHAPE"] and rows(cap=-5) == B.ERR["SHAPE"]
    assert rows(lda=32) == B.ERR["SHAPE"] and rows(ldc=8) == B.ERR["SHAPE"]
    assert rows(d_grp=p, n_groups=4, stride=256 * 64) == B.ERR["SHAPE"]    # all groups at once and a device row count
    assert rows(d_rows=None, d_grp=None, n_groups=4) == B.ERR["NULL"]
    assert b"as_op_gemm_rows" in B.lib.as_last_error(ctx.handle)
    assert B.lib.as_profile_only(ctx.handle, len(B.KERNEL_CLASSES)) == B.ERR["SHAPE"]
    assert B.lib.as_profile_only(ctx.handle, B.KERNEL_CLASSES.index("norm")) == 0
    assert B.lib.as_profile_only(ctx.handle, -1) == 0
    assert B.lib.as_profile_only(None, 0) == B.ERR["NULL"]
    ctx.close()
