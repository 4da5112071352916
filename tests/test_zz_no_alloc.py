"""The attention-backward entry point that allocates nothing (its scratch is a device array inside the
library) against the entry point that takes the scratch buffers from the caller: same kernels on the same
data, so the results must be the same bits.  Two calls in a row, the second on a smaller input (the array
keeps the first call's contents), then an input too large for the array."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def _inputs(seed, lens, Hq, Hkv, dh, dt):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(cu[-1])
    seg = np.searchsorted(cu, np.arange(n), side="right") - 1
    ss = torch.from_numpy(cu[seg].astype(np.int32)).cuda(); se = torch.from_numpy(cu[seg + 1].astype(np.int32)).cuda()
    qkv = torch.empty(n, (Hq + 2 * Hkv) * dh, dtype=torch.float32, device="cuda").normal_(0, 1.0, generator=g).to(dt)
    do = torch.empty(n, Hq * dh, dtype=torch.float32, device="cuda").normal_(0, 1.0, generator=g).to(dt)
    return qkv, do, ss, se


@pytest.mark.parametrize("bf16,Hq,Hkv,dh", [(True, 4, 2, 64), (True, 8, 2, 128), (False, 4, 4, 32)])
def test_static_scratch_entry_point_matches_the_workspace_one(bf16, Hq, Hkv, dh):
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[1].replace(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=dh)
    mode = B.AS_BF16 if bf16 else B.AS_FP32
    ctx = B.Context(B.make_config(sh, mode=mode))
    dt = torch.bfloat16 if bf16 else torch.float32
    for seed, lens in ((1, [300, 70, 129, 5, 257]), (2, [131, 64])):       # second call: fewer tokens, other boundaries
        qkv, do, ss, se = _inputs(seed, lens, Hq, Hkv, dh, dt)
        o, lse = ctx.op_attention_fwd(qkv, ss, mode=mode)
        want = ctx.op_attention_bwd(qkv, ss, se, o, lse, do, mode=mode)
        got = torch.full_like(qkv, float("nan"))
        ctx.op_attention_bwd(qkv, ss, se, o, lse, do, mode=mode, static=True, out=got)
        torch.cuda.synchronize()
        assert torch.isfinite(want.float()).all()
        assert torch.equal(got, want), (seed, (got.float() - want.float()).abs().max().item())


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    from paper_2503_22673_amd import binding as B
    sh = synth.CONFIGS[3]
    ctx = B.Context(B.make_config(sh))
    per_token = (6 * sh.n_q_heads + sh.n_kv_heads) * sh.head_dim * 2 + sh.n_q_heads * 4
    n = B.STATIC_SCRATCH_BYTES // per_token + 64                            # one tile of 64 tokens too many
    qkv, do, ss, se = _inputs(3, [n], sh.n_q_heads, sh.n_kv_heads, sh.head_dim, torch.bfloat16)
    o = torch.zeros(n, sh.n_q_heads * sh.head_dim, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(n, sh.n_q_heads, dtype=torch.float32, device="cuda")
    with pytest.raises(B.ASError) as e:
        ctx.op_attention_bwd(qkv, ss, se, o, lse, do, static=True)
    assert e.value.code == B.ERR["WORKSPACE"] and "scratch" in str(e.value)
