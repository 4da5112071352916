"""ctypes binding of libactionstudio.so: argument marshalling only.

Every step of the training path runs inside the library's HIP kernels; torch
is used to own device memory and to hand over the current stream.  There is
no fallback: if the shared library is missing, importing this module fails.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libactionstudio.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libactionstudio.so is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or paper_2503_22673_amd/build.py) first")
lib = C.CDLL(LIB_PATH)

AS_OK = 0
ERR = dict(NULL=-1, CONFIG=-2, SHAPE=-3, CU_SEQLENS=-4, TOKEN_RANGE=-5, ROLE=-6, TOO_LONG=-7, WORKSPACE=-8, HIP=-9)
AS_FP32, AS_BF16 = 0, 1
AS_LORA, AS_FULL = 0, 1
TARGETS = ("q", "k", "v", "o", "gate", "up", "down", "router")
N_TARGETS = 8
_WFIELDS = ("g1", "wq", "wk", "wv", "wo", "g2", "wgate", "wup", "wdown", "wrouter")
_AFIELDS = ("aq", "ak", "av", "ao", "agate", "aup", "adown")      # NF4 block maxima of wq .. wdown
_QUANT = dict(zip(("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"), _AFIELDS))
AS_W_DENSE, AS_W_NF4 = 0, 1
AS_PACK_NEXT_FIT, AS_PACK_BEST_FIT_DECREASING = 0, 1


class ModelConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("lora_rank", C.c_int32), ("lora_alpha", C.c_float), ("lora_targets", C.c_uint32),
                ("mode", C.c_int32), ("train_mode", C.c_int32), ("recompute", C.c_int32), ("weight_format", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in _WFIELDS + _AFIELDS]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("g_final", C.c_void_p), ("head", C.c_void_p),
                ("layers", C.POINTER(LayerWeights))]


class LayerLora(C.Structure):
    _fields_ = [("a", C.c_void_p * N_TARGETS), ("b", C.c_void_p * N_TARGETS)]


class Lora(C.Structure):
    _fields_ = [("layers", C.POINTER(LayerLora))]


class LayerWeightGrads(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in _WFIELDS]


class Grads(C.Structure):
    _fields_ = [("lora_layers", C.POINTER(LayerLora)), ("w_layers", C.POINTER(LayerWeightGrads)),
                ("embed", C.c_void_p), ("g_final", C.c_void_p), ("head", C.c_void_p)]


_vp, _i32, _i64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
lib.as_create.argtypes = [C.POINTER(_vp), C.POINTER(ModelConfig), C.c_int]
lib.as_destroy.argtypes = [_vp]
lib.as_destroy.restype = None
lib.as_last_error.argtypes = [_vp]
lib.as_last_error.restype = C.c_char_p
lib.as_workspace_bytes.argtypes = [_vp, _i64, _i64, C.POINTER(C.c_size_t)]
lib.as_pack.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp,
                        C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32), _vp, _vp]
lib.as_pack_policy.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp,
                               C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32), _vp, _vp, _vp]
lib.as_train_step.argtypes = [_vp, C.POINTER(Weights), C.POINTER(Lora), _vp, _vp, _vp, _i32, _vp, _vp, _i32, _i32,
                              _vp, _vp, _vp, C.POINTER(Grads), _vp, C.c_size_t, _vp]
lib.as_sequence_logps.argtypes = [_vp, C.POINTER(Weights), C.POINTER(Lora), _vp, _vp, _vp, _i32, _vp, _vp, _i32, _i32,
                                  _vp, _vp, C.c_size_t, _vp]
lib.as_dpo_step.argtypes = [_vp, C.POINTER(Weights), C.POINTER(Lora), _vp, _vp, _vp, _i32, _vp, _vp, _i32, _i32,
                            _vp, _i32, _vp, _f32, _vp, _vp, C.POINTER(Grads), _vp, C.c_size_t, _vp]
lib.as_adamw_update.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i64, _f32, _f32, _f32, _f32, _f32, _vp]
lib.as_op_gemm.argtypes = [_vp, C.c_int, C.c_int, _i64, _i64, _vp, _i64, _vp, _i64, _i64, _vp, _i64, _vp, _i64, _i64,
                           _f32, _vp, _i64, _vp, _i64, C.c_int, _vp, C.c_size_t, _vp]
GEMM_TAIL_SCRATCH_BYTES = 64 << 20
lib.as_op_gemm_rows.argtypes = [_vp, C.c_int, C.c_int, _i64, _i64, _vp, _i64, _vp, _i64, _i64, _f32, _vp, _i64, _vp, _i64, C.c_int,
                                _vp, _i64, _vp, C.c_int, C.c_int, _i64, _i64, _vp]
lib.as_op_rmsnorm_fwd.argtypes = [_vp, C.c_int, _i64, _i64, _vp, _vp, _f32, _vp, _vp, _vp]
lib.as_op_rmsnorm_bwd.argtypes = [_vp, C.c_int, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.as_op_attention_fwd.argtypes = [_vp, C.c_int, C.c_int, _i64, _vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _vp]
lib.as_op_attention_bwd.argtypes = [_vp, C.c_int, C.c_int, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp,
                                    _vp, _vp, _vp, _vp, _vp, _vp]
lib.as_op_head_loss_workspace.argtypes = [_vp, C.c_int, _i64, C.POINTER(C.c_size_t)]
lib.as_op_head_loss_workspace.restype = C.c_int
lib.as_op_head_loss.argtypes = [_vp, C.c_int, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
lib.as_op_head_loss.restype = C.c_int
lib.as_op_attention_bwd_static.argtypes = [_vp, C.c_int, C.c_int, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp,
                                           _vp, _vp, _vp, _vp]
lib.as_op_attention_bwd_static.restype = C.c_int
STATIC_SCRATCH_BYTES = 32 << 20
lib.as_probe_lds_feed.argtypes = [_vp, _i32, _vp, C.c_size_t, _i32, _i32, _vp, C.POINTER(C.c_double), _vp]
lib.as_probe_lds_feed.restype = C.c_int
lib.as_probe_mfma_peak.argtypes = [_vp, _i32, _i32, _vp, C.POINTER(C.c_double), _vp]
lib.as_probe_mfma_peak.restype = C.c_int
lib.as_profile.argtypes = [_vp, C.c_int]
lib.as_profile_only.argtypes = [_vp, C.c_int]
lib.as_profile_read.argtypes = [_vp, C.c_int, C.POINTER(_i64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
KERNEL_CLASSES = ("gemm_mfma_256", "gemm_mfma_skinny", "gemm_fma", "gemm_devrows", "attn_fwd", "attn_bwd", "transpose",
                  "norm", "swiglu", "rope", "ce", "lora_grad", "gemm_grouped", "moe", "gemm_mfma_rs")
for _n in ("as_profile", "as_profile_read", "as_create", "as_workspace_bytes", "as_pack", "as_train_step", "as_adamw_update", "as_op_gemm",
           "as_op_rmsnorm_fwd", "as_op_rmsnorm_bwd", "as_op_attention_fwd", "as_op_attention_bwd", "as_nf4_quantize", "as_nf4_dequantize", "as_sequence_logps", "as_dpo_step", "as_pack_policy", "as_op_gemm_rows", "as_profile_only"):
    getattr(lib, _n).restype = C.c_int

EXPORTS = ("as_op_head_loss", "as_op_head_loss_workspace", "as_op_attention_bwd_static", "as_probe_lds_feed", "as_probe_mfma_peak", "as_profile", "as_profile_read", "as_create", "as_destroy", "as_last_error", "as_workspace_bytes", "as_pack", "as_train_step",
           "as_adamw_update", "as_op_gemm", "as_op_rmsnorm_fwd", "as_op_rmsnorm_bwd", "as_op_attention_fwd",
           "as_op_attention_bwd", "as_nf4_quantize", "as_nf4_dequantize", "as_sequence_logps", "as_dpo_step", "as_pack_policy", "as_op_gemm_rows", "as_profile_only")


class ASError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("actionstudio error %d: %s" % (code, msg))
        self.code = code


def make_config(sh, mode=None, train_mode=None, recompute=None, weight_format=AS_W_DENSE):
    """sh: any object with the attribute names of synth.Shape."""
    full = bool(getattr(sh, "full_ft", False)) if train_mode is None else train_mode == AS_FULL
    mask = 0
    if not full:
        for t in sh.lora_targets:
            mask |= 1 << TARGETS.index(t)
    if mode is None:
        mode = AS_BF16 if sh.bf16 else AS_FP32
    if recompute is None:
        recompute = int(getattr(sh, "recompute", 0))
    return ModelConfig(C.sizeof(ModelConfig), sh.n_layers, sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
                       sh.ffn, sh.vocab, sh.n_experts, sh.top_k, sh.rms_eps, sh.rope_base,
                       0 if full else sh.lora_rank, 0.0 if full else sh.lora_alpha, mask, mode,
                       AS_FULL if full else AS_LORA, recompute, weight_format)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    def __init__(self, cfg, device=0):
        self.cfg = cfg
        self.handle = C.c_void_p()
        rc = lib.as_create(C.byref(self.handle), C.byref(cfg), device)
        if rc:
            raise ASError(rc, lib.as_last_error(None).decode())
        self.device = device
        self.mode = cfg.mode
        self.dtype = torch.float32 if cfg.mode == AS_FP32 else torch.bfloat16

    def close(self):
        if self.handle:
            lib.as_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc):
        if rc:
            raise ASError(rc, lib.as_last_error(self.handle).decode())

    def workspace_bytes(self, max_rows, row_len):
        out = C.c_size_t()
        self.check(lib.as_workspace_bytes(self.handle, max_rows, row_len, C.byref(out)))
        return out.value

    def probe_lds_feed(self, loads_in_flight, span_bytes, iters=2000, blocks=256, buf=None):
        dev = torch.device("cuda", self.device)
        if buf is None:
            buf = torch.ones(span_bytes, dtype=torch.uint8, device=dev)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        out = C.c_double()
        self.check(lib.as_probe_lds_feed(self.handle, loads_in_flight, _ptr(buf), span_bytes, iters, blocks, _ptr(sink),
                                         C.byref(out), _stream()))
        return out.value

    def probe_mfma_peak(self, iters=20000, blocks=2048):
        sink = torch.zeros(1, dtype=torch.float32, device=torch.device("cuda", self.device))
        out = C.c_double()
        self.check(lib.as_probe_mfma_peak(self.handle, iters, blocks, _ptr(sink), C.byref(out), _stream()))
        return out.value

    def profile(self, enable, only=None):
        """only: name of the one kernel class to bracket (None: every class)"""
        if enable:
            self.check(lib.as_profile(self.handle, 0))
            self.check(lib.as_profile_only(self.handle, -1 if only is None else KERNEL_CLASSES.index(only)))
        self.check(lib.as_profile(self.handle, int(enable)))

    def profile_read(self):
        """{class name: (launches, total ms, total flops)} for the launches recorded so far."""
        out = {}
        for i, name in enumerate(KERNEL_CLASSES):
            n, ms, fl = _i64(), C.c_double(), C.c_double()
            self.check(lib.as_profile_read(self.handle, i, C.byref(n), C.byref(ms), C.byref(fl)))
            out[name] = (n.value, ms.value, fl.value)
        return out

    # ---------------------------------------------------------------- pack
    def pack(self, turn_tokens, turn_offsets, turn_roles, traj_offsets, row_len, max_rows, pad_id=0,
             truncate=True, outputs=None, policy=None):
        """Host numpy arrays in; device tensors (tokens, cu_seqlens, loss_mask) out.  policy None: as_pack (next
        fit); AS_PACK_NEXT_FIT / AS_PACK_BEST_FIT_DECREASING: as_pack_policy, which also reports traj_row."""
        tt = np.ascontiguousarray(turn_tokens, dtype=np.int32)
        to = np.ascontiguousarray(turn_offsets, dtype=np.int32)
        tr = np.ascontiguousarray(turn_roles, dtype=np.uint8)
        jo = np.ascontiguousarray(traj_offsets, dtype=np.int32)
        n_traj = len(jo) - 1
        if outputs is None:
            dev = torch.device("cuda", self.device)
            n_out = max(1, max_rows * row_len)
            outputs = (torch.empty(n_out, dtype=torch.int32, device=dev),
                       torch.empty(n_traj + max_rows + 1, dtype=torch.int32, device=dev),
                       torch.empty(n_out, dtype=torch.uint8, device=dev))
        tok, cu, msk = outputs
        nr, ns, nc = _i32(), _i32(), _i32()
        skip = np.zeros(max(1, n_traj + max(max_rows, 0)), dtype=np.uint8)
        hp = lambda a: a.ctypes.data_as(C.c_void_p) if a.size else None
        st = _stream() if tok is not None and tok.is_cuda else None
        traj_row = None
        if policy is None:
            self.check(lib.as_pack(self.handle, hp(tt), hp(to), hp(tr), hp(jo), n_traj, row_len, max_rows, pad_id,
                                   int(truncate), _ptr(tok), _ptr(cu), _ptr(msk), C.byref(nr), C.byref(ns), C.byref(nc),
                                   hp(skip), st))
        else:
            traj_row = np.full(max(1, n_traj), -1, dtype=np.int32)
            self.check(lib.as_pack_policy(self.handle, hp(tt), hp(to), hp(tr), hp(jo), n_traj, row_len, max_rows, pad_id,
                                          int(truncate), int(policy), _ptr(tok), _ptr(cu), _ptr(msk), C.byref(nr), C.byref(ns),
                                          C.byref(nc), hp(skip), hp(traj_row), st))
            traj_row = traj_row[:n_traj]
        n = nr.value * row_len
        return dict(tokens=tok[:n], cu_seqlens=cu[:ns.value + 1], loss_mask=msk[:n], n_rows=nr.value,
                    n_segments=ns.value, n_traj_consumed=nc.value, seg_skip=skip[:ns.value].copy(), traj_row=traj_row)

    # ----------------------------------------------------------- train step
    def train_step(self, model, tokens, cu_seqlens, h_cu_seqlens, loss_mask, n_rows, row_len, workspace, out=None,
                   seg_skip=None):
        """model: DeviceModel.  Returns dict of device scalars (loss, loss_sum, count)."""
        dev = tokens.device
        if out is None:
            out = dict(loss=torch.zeros(1, dtype=torch.float32, device=dev),
                       loss_sum=torch.zeros(1, dtype=torch.float32, device=dev),
                       count=torch.zeros(1, dtype=torch.int32, device=dev))
        hcu = np.ascontiguousarray(h_cu_seqlens, dtype=np.int32)
        hskip = None
        if seg_skip is not None:
            hskip = np.ascontiguousarray(seg_skip, dtype=np.uint8)
            assert len(hskip) == len(hcu) - 1
        self.check(lib.as_train_step(self.handle, C.byref(model.c_weights),
                                     C.byref(model.c_lora) if model.c_lora is not None else None,
                                     _ptr(tokens), _ptr(cu_seqlens), hcu.ctypes.data_as(C.c_void_p), len(hcu) - 1,
                                     hskip.ctypes.data_as(C.c_void_p) if hskip is not None else None, _ptr(loss_mask), n_rows, row_len, _ptr(out["loss"]), _ptr(out["loss_sum"]),
                                     _ptr(out["count"]), C.byref(model.c_grads), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))
        return out

    # ------------------------------------------------- preference learning
    @staticmethod
    def _skip(seg_skip, hcu):
        if seg_skip is None:
            return None, None
        hskip = np.ascontiguousarray(seg_skip, dtype=np.uint8)
        assert len(hskip) == len(hcu) - 1
        return hskip, hskip.ctypes.data_as(C.c_void_p)

    def sequence_logps(self, model, tokens, cu_seqlens, h_cu_seqlens, loss_mask, n_rows, row_len, workspace,
                       seg_skip=None, adapters=True):
        """Per-segment sums of log p over the targets (device float [n_segments]); adapters=False: base model."""
        hcu = np.ascontiguousarray(h_cu_seqlens, dtype=np.int32)
        hskip, pskip = self._skip(seg_skip, hcu)
        logp = torch.empty(len(hcu) - 1, dtype=torch.float32, device=tokens.device)
        lora = C.byref(model.c_lora) if (adapters and model.c_lora is not None) else None
        self.check(lib.as_sequence_logps(self.handle, C.byref(model.c_weights), lora, _ptr(tokens), _ptr(cu_seqlens),
                                         hcu.ctypes.data_as(C.c_void_p), len(hcu) - 1, pskip, _ptr(loss_mask), n_rows, row_len,
                                         _ptr(logp), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
        return logp

    def dpo_step(self, model, tokens, cu_seqlens, h_cu_seqlens, loss_mask, n_rows, row_len, workspace, pairs, ref_logp,
                 beta, seg_skip=None):
        """pairs: [P, 2] (chosen, rejected) segment indices.  Returns dict(stats = device float[3]: loss, margin,
        accuracy; logp = device float [n_segments]); gradients land in the model's gradient buffers."""
        hcu = np.ascontiguousarray(h_cu_seqlens, dtype=np.int32)
        hskip, pskip = self._skip(seg_skip, hcu)
        hp = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        out = dict(stats=torch.zeros(3, dtype=torch.float32, device=tokens.device),
                   logp=torch.empty(len(hcu) - 1, dtype=torch.float32, device=tokens.device))
        self.check(lib.as_dpo_step(self.handle, C.byref(model.c_weights),
                                   C.byref(model.c_lora) if model.c_lora is not None else None, _ptr(tokens),
                                   _ptr(cu_seqlens), hcu.ctypes.data_as(C.c_void_p), len(hcu) - 1, pskip, _ptr(loss_mask),
                                   n_rows, row_len, hp.ctypes.data_as(C.c_void_p) if len(hp) else None, len(hp), _ptr(ref_logp), beta,
                                   _ptr(out["stats"]), _ptr(out["logp"]), C.byref(model.c_grads), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))
        return out

    # ---------------------------------------------------------------- AdamW
    def adamw_update(self, masters, lowps, grads, ms, vs, apply_wd, step, lr, beta1, beta2, eps, weight_decay):
        n = len(masters)
        arr = lambda ts: (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in ts])
        numel = (C.c_int64 * n)(*[t.numel() for t in masters])
        wd = (C.c_uint8 * n)(*[int(bool(x)) for x in apply_wd])
        self.check(lib.as_adamw_update(self.handle, arr(masters), arr(lowps) if lowps is not None else None,
                                       arr(grads), arr(ms), arr(vs), numel, wd, n, step, lr, beta1, beta2, eps,
                                       weight_decay, _stream()))

    # ------------------------------------------------------- building blocks
    def op_gemm(self, A1, B1, A2=None, B2=None, alpha=1.0, R=None, out_f32=False, variant=0, mode=None, tail_scratch=None):
        """tail_scratch: uint8 device tensor of GEMM_TAIL_SCRATCH_BYTES, lets the kernel split its last round of tiles"""
        mode = self.mode if mode is None else mode
        M, K1 = A1.shape
        N = B1.shape[0]
        Cm = torch.empty(M, N, dtype=torch.float32 if out_f32 else A1.dtype, device=A1.device)
        K2 = A2.shape[1] if A2 is not None else 0
        self.check(lib.as_op_gemm(self.handle, mode, variant, M, N, _ptr(A1), A1.stride(0), _ptr(B1), B1.stride(0), K1,
                                  _ptr(A2), A2.stride(0) if A2 is not None else 0, _ptr(B2),
                                  B2.stride(0) if B2 is not None else 0, K2, alpha, _ptr(R),
                                  R.stride(0) if R is not None else 0, _ptr(Cm), Cm.stride(0), int(out_f32), _ptr(tail_scratch),
                                  tail_scratch.numel() if tail_scratch is not None else 0, _stream()))
        return Cm

    def op_gemm_rows(self, A, Bm, Cm, alpha=1.0, R=None, d_rows=None, row_off=0, d_group_off=None, group=0, rows_cap=0, M=None,
                     n_groups=0, variant=0, mode=None):
        """Cm (caller's buffer, float32 or A's type) receives the live rows of alpha * A Bm^T (+ R); the other rows stay as they are."""
        mode = self.mode if mode is None else mode
        M = A.shape[0] if M is None else M
        # n_groups > 0: Bm is [n_groups, N, K], the stacked matrices of the groups
        N, ldb, stride = (Bm.shape[1], Bm.stride(1), Bm.stride(0)) if n_groups else (Bm.shape[0], Bm.stride(0), 0)
        self.check(lib.as_op_gemm_rows(self.handle, mode, variant, M, N, _ptr(A), A.stride(0), _ptr(Bm), ldb, A.shape[1],
                                       alpha, _ptr(R), R.stride(0) if R is not None else 0, _ptr(Cm), Cm.stride(0),
                                       int(Cm.dtype == torch.float32), _ptr(d_rows), row_off, _ptr(d_group_off), group, n_groups, stride,
                                       rows_cap, _stream()))
        return Cm

    def op_head_loss(self, hf, head, labels, count, row_w=None, mode=None):
        """hf [rows, d] (rows a multiple of 256 at least the row capacity of labels), head [V, d], labels int32 [n_rows], count
        device int32[1].  Returns (loss_rows float [n_rows], dhf like hf); rows at or past the count are left as they were (zero)."""
        mode = self.mode if mode is None else mode
        n_rows = labels.numel()
        assert hf.shape[0] >= (n_rows + 255) // 256 * 256
        need = C.c_size_t()
        self.check(lib.as_op_head_loss_workspace(self.handle, mode, n_rows, C.byref(need)))
        ws = torch.empty(need.value, dtype=torch.uint8, device=hf.device)
        loss = torch.zeros(n_rows, dtype=torch.float32, device=hf.device)
        dhf = torch.zeros_like(hf)
        self.check(lib.as_op_head_loss(self.handle, mode, n_rows, _ptr(hf), _ptr(head), _ptr(labels), _ptr(count), _ptr(row_w), _ptr(loss),
                                       _ptr(dhf), _ptr(ws), need.value, _stream()))
        return loss, dhf

    def nf4_quantize(self, w):
        """w: device tensor (float32 or bfloat16), numel a multiple of 64 -> (packed codes uint8 [numel/2], absmax float32 [numel/64])."""
        w = w.contiguous()
        mode = AS_FP32 if w.dtype == torch.float32 else AS_BF16
        codes = torch.empty(w.numel() // 2, dtype=torch.uint8, device=w.device)
        absmax = torch.empty(w.numel() // 64, dtype=torch.float32, device=w.device)
        self.check(lib.as_nf4_quantize(self.handle, mode, _ptr(w), C.c_int64(w.numel()), _ptr(codes), _ptr(absmax), _stream()))
        return codes, absmax

    def nf4_dequantize(self, codes, absmax, dtype):
        mode = AS_FP32 if dtype == torch.float32 else AS_BF16
        out = torch.empty(codes.numel() * 2, dtype=dtype, device=codes.device)
        self.check(lib.as_nf4_dequantize(self.handle, mode, _ptr(codes), _ptr(absmax), C.c_int64(out.numel()), _ptr(out), _stream()))
        return out

    def op_rmsnorm_fwd(self, x, g, eps, mode=None):
        mode = self.mode if mode is None else mode
        n, d = x.shape
        y = torch.empty_like(x)
        rstd = torch.empty(n, dtype=torch.float32, device=x.device)
        self.check(lib.as_op_rmsnorm_fwd(self.handle, mode, n, d, _ptr(x), _ptr(g), eps, _ptr(y), _ptr(rstd), _stream()))
        return y, rstd

    def op_rmsnorm_bwd(self, dy, x, g, rstd, add=None, mode=None):
        mode = self.mode if mode is None else mode
        n, d = x.shape
        dx = torch.empty_like(x)
        self.check(lib.as_op_rmsnorm_bwd(self.handle, mode, n, d, _ptr(dy), _ptr(x), _ptr(g), _ptr(rstd), _ptr(add),
                                         _ptr(dx), _stream()))
        return dx

    def op_attention_fwd(self, qkv, seg_start, variant=0, mode=None):
        """qkv [n, (Hq + 2 Hkv) * dh] packed side by side."""
        mode = self.mode if mode is None else mode
        c = self.cfg
        n = qkv.shape[0]
        D, Dkv = c.n_q_heads * c.head_dim, c.n_kv_heads * c.head_dim
        es = qkv.element_size()
        o = torch.empty(n, D, dtype=qkv.dtype, device=qkv.device)
        lse = torch.empty(n, c.n_q_heads, dtype=torch.float32, device=qkv.device)
        base = qkv.data_ptr()
        n64 = (n + 63) // 64 * 64
        ts = torch.empty(Dkv * n64, dtype=qkv.dtype, device=qkv.device)
        self.check(lib.as_op_attention_fwd(self.handle, mode, variant, n, _ptr(seg_start), C.c_void_p(base), qkv.stride(0),
                                           C.c_void_p(base + D * es), C.c_void_p(base + (D + Dkv) * es), qkv.stride(0),
                                           _ptr(o), _ptr(lse), _ptr(ts), _stream()))
        return o, lse

    def op_attention_bwd(self, qkv, seg_start, seg_end, o, lse, d_o, variant=0, mode=None, static=False, out=None):
        """static=True: the entry point that allocates nothing (scratch inside the library); out: caller's dqkv buffer."""
        mode = self.mode if mode is None else mode
        c = self.cfg
        n = qkv.shape[0]
        D, Dkv = c.n_q_heads * c.head_dim, c.n_kv_heads * c.head_dim
        es = qkv.element_size()
        dqkv = torch.empty_like(qkv) if out is None else out
        if static:
            b, g = qkv.data_ptr(), dqkv.data_ptr()
            self.check(lib.as_op_attention_bwd_static(self.handle, mode, variant, n, _ptr(seg_start), _ptr(seg_end), C.c_void_p(b),
                                                      qkv.stride(0), C.c_void_p(b + D * es), C.c_void_p(b + (D + Dkv) * es),
                                                      qkv.stride(0), _ptr(o), _ptr(lse), _ptr(d_o), C.c_void_p(g),
                                                      C.c_void_p(g + D * es), C.c_void_p(g + (D + Dkv) * es), _stream()))
            return dqkv
        delta = torch.empty(n, c.n_q_heads, dtype=torch.float32, device=qkv.device)
        b, g = qkv.data_ptr(), dqkv.data_ptr()
        n64 = (n + 63) // 64 * 64
        ts = torch.empty((6 * D + Dkv) * n64, dtype=qkv.dtype, device=qkv.device)
        self.check(lib.as_op_attention_bwd(self.handle, mode, variant, n, _ptr(seg_start), _ptr(seg_end), C.c_void_p(b),
                                           qkv.stride(0), C.c_void_p(b + D * es), C.c_void_p(b + (D + Dkv) * es),
                                           qkv.stride(0), _ptr(o), _ptr(lse), _ptr(d_o), C.c_void_p(g),
                                           C.c_void_p(g + D * es), C.c_void_p(g + (D + Dkv) * es), _ptr(delta), _ptr(ts), _stream()))
        return dqkv


class DeviceModel:
    """Owns the device tensors of weights, adapters and gradients and the
    pointer tables the C interface takes."""

    def __init__(self, ctx, params, lora=None):
        """params / lora: the nested dict / list layout of synth.weights and
        synth.lora_weights, holding numpy arrays or torch tensors."""
        self.ctx = ctx
        cfg = ctx.cfg
        dev = torch.device("cuda", ctx.device)
        wd = ctx.dtype
        full = cfg.train_mode == AS_FULL

        def up(x, dt):
            if isinstance(x, torch.Tensor):
                return x.to(device=dev, dtype=dt).contiguous()
            return torch.from_numpy(np.ascontiguousarray(x)).to(device=dev, dtype=dt).contiguous()

        self.embed, self.head, self.g_final = up(params["embed"], wd), up(params["head"], wd), up(params["g_final"], wd)
        def up_w(k, v):                      # NF4: codes stay uint8, block maxima float
            if cfg.weight_format == AS_W_NF4 and k in _QUANT:
                return up(v, torch.uint8)
            return up(v, torch.float32 if k in _AFIELDS else wd)

        self.layers = [{k: up_w(k, v) for k, v in W.items()} for W in params["layers"]]
        L = cfg.n_layers
        self._lw = (LayerWeights * L)()
        for l, W in enumerate(self.layers):
            for f in _WFIELDS + _AFIELDS:
                setattr(self._lw[l], f, W[f].data_ptr() if f in W else None)
        self.c_weights = Weights(self.embed.data_ptr(), self.g_final.data_ptr(), self.head.data_ptr(), self._lw)
        self.c_lora = None
        self.lora, self.lora_grads, self.w_grads = None, None, None
        self.c_grads = Grads()
        if not full:
            self.lora = [{k: (up(A, torch.float32), up(B, torch.float32)) for k, (A, B) in Lr.items()} for Lr in lora]
            self.lora_grads = [{k: (torch.zeros_like(A), torch.zeros_like(B)) for k, (A, B) in Lr.items()} for Lr in self.lora]
            self._ll = (LayerLora * L)()
            self._lg = (LayerLora * L)()
            for l in range(L):
                for i, t in enumerate(TARGETS):
                    if t in self.lora[l]:
                        self._ll[l].a[i], self._ll[l].b[i] = self.lora[l][t][0].data_ptr(), self.lora[l][t][1].data_ptr()
                        self._lg[l].a[i], self._lg[l].b[i] = self.lora_grads[l][t][0].data_ptr(), self.lora_grads[l][t][1].data_ptr()
            self.c_lora = Lora(self._ll)
            self.c_grads.lora_layers = self._lg
        else:
            f32 = torch.float32
            self.w_grads = dict(embed=torch.zeros(self.embed.shape, dtype=f32, device=dev),
                                head=torch.zeros(self.head.shape, dtype=f32, device=dev),
                                g_final=torch.zeros(self.g_final.shape, dtype=f32, device=dev),
                                layers=[{k: torch.zeros(v.shape, dtype=f32, device=dev) for k, v in W.items()}
                                        for W in self.layers])
            self._wg = (LayerWeightGrads * L)()
            for l, W in enumerate(self.w_grads["layers"]):
                for f in _WFIELDS:
                    setattr(self._wg[l], f, W[f].data_ptr() if f in W else None)
            self.c_grads.w_layers = self._wg
            self.c_grads.embed = self.w_grads["embed"].data_ptr()
            self.c_grads.head = self.w_grads["head"].data_ptr()
            self.c_grads.g_final = self.w_grads["g_final"].data_ptr()
