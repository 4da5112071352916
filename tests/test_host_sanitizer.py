"""The host half of the C interface (configuration checks, packing plan, segment-table check: csrc/host_logic.cpp)
built with g++ -fsanitize=address,undefined and driven with valid and invalid inputs.  Valid packing cases are
checked against the float64 reference's packer; invalid ones must come back with the right status and without a
sanitizer report (every input array is a heap block of exactly its length)."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import synth
from helpers import random_trajs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_22673_amd", "csrc")
ERR = dict(NULL=-1, CONFIG=-2, SHAPE=-3, CU_SEQLENS=-4, TOKEN_RANGE=-5, ROLE=-6, TOO_LONG=-7)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "host_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, os.path.join(CSRC, "host_logic.cpp"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr

    def run(text):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
        p = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=120)
        assert p.returncode == 0 and "ERROR" not in p.stderr and "runtime error" not in p.stderr, (p.returncode, p.stderr[-2000:])
        return p.stdout.splitlines()
    return run


def pack_case(trajs, vocab, T, max_rows, truncate=1, policy=0, flat=None):
    tt, to, tr, jo = synth.flatten_trajectories(trajs) if flat is None else flat
    hdr = "pack %d %d %d %d %d %d %d %d" % (vocab, T, max_rows, truncate, policy, len(jo) - 1, len(tr), len(tt))
    return "\n".join([hdr, " ".join(map(str, jo)), " ".join(map(str, to)), " ".join(map(str, tr)), " ".join(map(str, tt))]) + "\n"


def parse_pack(lines):
    d = {}
    for l in lines:
        k, *v = l.split()
        d[k] = v
    return d


@pytest.mark.parametrize("policy", [0, 1])
def test_valid_packing_cases_match_the_reference_packer(driver, policy):
    for seed in range(6):
        vocab, T, rows = 50, (64, 37, 128)[seed % 3], (3, 5, 2)[seed % 3]
        trajs = random_trajs(seed, 9, vocab, turn_lo=1, turn_hi=30, turns=(1, 5))
        if seed == 2:
            trajs.insert(1, [])                                             # an empty trajectory
            trajs.insert(3, [(1, np.zeros(0, dtype=np.int32))])             # a trajectory of one empty turn
        out = parse_pack(driver(pack_case(trajs, vocab, T, rows, policy=policy)))
        assert out["rc"] == ["0"]
        ref = oracle.pack(trajs, T, rows, pad_id=-1, policy="best_fit_decreasing" if policy else "next_fit")
        n = ref["n_rows"] * T
        assert int(out["rows"][0]) == ref["n_rows"] and int(out["rows"][2]) == ref["n_traj_consumed"]
        assert list(map(int, out["cu"][:])) == ref["cu_seqlens"].tolist()
        assert list(map(int, out.get("tokens", []))) == ref["tokens"][:n].tolist()
        assert list(map(int, out.get("mask", []))) == ref["loss_mask"][:n].astype(int).tolist()
        cu, mask = ref["cu_seqlens"], ref["loss_mask"]
        assert list(map(int, out.get("skip", []))) == [int(not mask[a:b].any()) for a, b in zip(cu[:-1], cu[1:])]


def test_invalid_packing_inputs_are_refused_without_reading_out_of_bounds(driver):
    trajs = random_trajs(1, 4, 50, turn_lo=3, turn_hi=9)
    tt, to, tr, jo = synth.flatten_trajectories(trajs)
    cases = []
    def add(expect, **kw):
        flat = [a.copy() for a in (tt, to, tr, jo)]
        args = dict(vocab=50, T=64, max_rows=4, truncate=1, policy=0)
        for k, v in kw.items():
            if k in args: args[k] = v
            else: v(flat)
        cases.append((expect, pack_case(None, args["vocab"], args["T"], args["max_rows"], args["truncate"], args["policy"], flat=tuple(flat))))
    add("SHAPE", T=0)
    add("SHAPE", max_rows=-1)
    add("SHAPE", policy=7)
    add("SHAPE", T=1 << 20, max_rows=1 << 12)                                # rows * row_len beyond int32
    add("SHAPE", f=lambda a: a[3].__setitem__(0, 1))                         # trajectory offsets not starting at 0
    add("SHAPE", f=lambda a: a[3].__setitem__(2, a[3][1] - 1))               # decreasing trajectory offsets
    add("SHAPE", f=lambda a: a[1].__setitem__(3, a[1][2] - 1))               # decreasing turn offsets
    add("ROLE", f=lambda a: a[2].__setitem__(1, 4))
    add("TOKEN_RANGE", f=lambda a: a[0].__setitem__(5, 50))
    add("TOKEN_RANGE", f=lambda a: a[0].__setitem__(0, -1))
    add("TOO_LONG", T=8, truncate=0)
    out = driver("".join(c for _, c in cases))
    rcs = [int(l.split()[1]) for l in out if l.startswith("rc ")]
    assert rcs == [ERR[e] for e, _ in cases], list(zip(rcs, [e for e, _ in cases]))
    # no trajectories at all, and zero rows asked for
    out = parse_pack(driver(pack_case([], 50, 16, 2)))
    assert out["rc"] == ["0"] and out["rows"][0] == "0" and out["cu"] == ["0"]
    out = parse_pack(driver(pack_case(trajs, 50, 64, 0)))
    assert out["rc"] == ["0"] and out["rows"][0] == "0"


def test_segment_table_check(driver):
    ok = "cu 3 128 64\n0 10 64 128\n"
    bad = ["cu 0 128 64\n0\n", "cu 3 128 64\n1 10 64 128\n", "cu 3 128 64\n0 10 64 127\n", "cu 3 128 64\n0 10 10 128\n",
           "cu 2 128 64\n0 70 128\n", "cu 3 128 64\n0 64 60 128\n"]
    out = driver(ok + "".join(bad))
    assert out[0] == "rc 0 max_seg 64"
    assert [l.split()[1] for l in out[1:]] == [str(ERR["CU_SEQLENS"])] * len(bad)


def test_configuration_check(driver):
    base = [0, 2, 128, 4, 4, 32, 344, 1024, 0, 0, 1e-5, 1e4, 8, 16.0, 15, 0, 0, 0, 0]
    def cfg(**kw):
        names = ["struct_size", "n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab", "n_experts", "top_k",
                 "rms_eps", "rope_base", "lora_rank", "lora_alpha", "lora_targets", "mode", "train_mode", "recompute", "weight_format"]
        v = list(base)
        for k, x in kw.items(): v[names.index(k)] = x
        return "cfg " + " ".join(str(x) for x in v) + "\n"
    good = [cfg(), cfg(train_mode=1, lora_rank=0, lora_targets=0), cfg(n_experts=8, top_k=2, lora_targets=0x8f), cfg(weight_format=1, ffn=384, head_dim=64)]
    bad = [cfg(struct_size=12), cfg(n_layers=0), cfg(n_kv_heads=3), cfg(head_dim=48), cfg(mode=2), cfg(rms_eps=0.0), cfg(lora_rank=0),
           cfg(lora_rank=300), cfg(lora_targets=0), cfg(lora_targets=0x80), cfg(n_experts=8, top_k=1), cfg(n_experts=8, top_k=2, lora_targets=0x10),
           cfg(train_mode=1), cfg(recompute=3), cfg(weight_format=2), cfg(weight_format=1, ffn=344)]
    out = driver("".join(good) + "".join(bad))
    assert out == ["rc 0"] * len(good) + ["rc %d" % ERR["CONFIG"]] * len(bad), out
