"""ctypes binding of libzoqat.so -- argument marshalling only.

Every function mirrors the C entry point of the same name in include/zoqat.h.  torch is used
for device memory and streams; every step of the path runs inside the HIP library.  The
module raises at import if the library has not been built (there is no CPU fallback)."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzoqat.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libzoqat.so is not built; run `python -c 'import __graft_entry__ as g; g.build()'` first")
_lib = C.CDLL(LIB_PATH)

ZO_OK = 0
STATUS = {0: "ZO_OK", 1: "ZO_EINVAL", 2: "ZO_ESHAPE", 3: "ZO_EALIGN", 4: "ZO_EHIP", 5: "ZO_EUNSUPPORTED", 6: "ZO_EWORKSPACE"}
ARCH_LINEAR, ARCH_LLAMA, ARCH_OPT = 0, 1, 2
ACT_FP32, ACT_BF16 = 0, 1
MASTER_F32, MASTER_F16 = 0, 1
ROUTE_FUSED_SMALL_M, ROUTE_FUSED_INT4, ROUTE_SWIGLU_IN_GEMM, ROUTE_ROPE_IN_GEMM, ROUTE_CE_IN_GEMM, ROUTE_GEMM_SPLIT_K, ROUTE_INT8_MMA = 1, 2, 4, 8, 16, 32, 64

EXPORTS = ["zo_num_params", "zo_param_numel", "zo_workspace_bytes", "zo_init", "zo_destroy", "zo_last_error",
           "zo_forward_quant", "zo_step", "zo_update", "zo_probe_mfma_only", "zo_debug_philox_u32", "zo_debug_normal", "zo_update_tensor",
           "zo_debug_quant_weight", "zo_debug_quant_act", "zo_linear_scratch_bytes", "zo_linear_fakequant",
           "zo_gemm_nt", "zo_debug_buffer", "zo_profile_begin", "zo_profile_end", "zo_attention_causal",
           "zo_attention_scratch_bytes", "zo_pack_weight_int4", "zo_attach_frozen_int4", "zo_linear_frozen_int4", "zo_gemm_nt_fused", "zo_init_learned_params", "zo_step_groups", "zo_update_groups",
           "zo_debug_quant_weight_learned", "zo_debug_smooth_bias", "zo_linear_fakequant_fused", "zo_linear_fused_scratch_bytes",
           "zo_step_multi", "zo_update_multi", "zo_lr_linear_decay", "zo_update_tensor_f16", "zo_master_bytes", "zo_linear_frozen_int4_fused", "zo_linear_frozen_fused_scratch_bytes", "zo_gemm_nt_swiglu", "zo_debug_routes", "zo_gemm_nt_ce", "zo_gemm_nt_ce_scratch_bytes", "zo_profile_begin_mask",
           "zo_gemm_nt_splitk_ranges", "zo_gemm_nt_splitk_scratch_bytes", "zo_gemm_nt_fused_splitk",
           "zo_gemm_nt_splitk_static_max_bytes", "zo_gemm_nt_fused_splitk_static",
           "zo_linear_mma_scratch_bytes", "zo_linear_fakequant_mma",
           "zo_kv_cache_bytes", "zo_prefill", "zo_decode", "zo_generate_greedy", "zo_linear_frozen_int4_token"]
PROF_NAMES = ["gemm", "weight_quant", "act_quant", "attention", "update", "other", "fused_linear", "fused_int4_linear"]


class zo_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("arch", "n_layers", "d_model", "n_heads", "d_ffn", "vocab", "max_seq",
                                         "w_bits", "w_group", "a_bits", "a_sym", "act_dtype", "lightweight",
                                         "learn_clip", "learn_smooth", "no_fused", "master_dtype", "master_round", "mma")]


class zo_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("numel", C.c_int64), ("trainable", C.c_int32), ("reserved", C.c_int32)]


class ZoError(RuntimeError):
    def __init__(self, status, where, detail=""):
        self.status = status
        super().__init__("%s returned %s%s" % (where, STATUS.get(status, status), (": " + detail) if detail else ""))


_vp, _i32, _i64, _u64, _f32, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
_lib.zo_num_params.argtypes = [C.POINTER(zo_config)]
_lib.zo_num_params.restype = _i32
_lib.zo_param_numel.argtypes = [C.POINTER(zo_config), _i32]
_lib.zo_param_numel.restype = _i64
_lib.zo_workspace_bytes.argtypes = [C.POINTER(zo_config), _i32, _i32]
_lib.zo_workspace_bytes.restype = _sz
_lib.zo_init.argtypes = [C.POINTER(zo_config), C.POINTER(zo_tensor), _i32, _vp, _sz, _i32, _i32, _vp, C.POINTER(_vp)]
_lib.zo_destroy.argtypes = [_vp]
_lib.zo_last_error.argtypes = [_vp]
_lib.zo_last_error.restype = C.c_char_p
_lib.zo_forward_quant.argtypes = [_vp, _vp, _vp, _i32, _i32, _u64, _f32, _vp]
_lib.zo_step.argtypes = [_vp, _vp, _vp, _i32, _i32, _u64, _f32, _f32, _vp]
_lib.zo_update.argtypes = [_vp, _u64, _vp, _f32]
_lib.zo_debug_philox_u32.argtypes = [_u64, _i32, _i64, _vp, _vp]
_lib.zo_probe_mfma_only.argtypes = [_vp, _i32, _i32, _i32, _vp]
_lib.zo_debug_normal.argtypes = [_u64, _i32, _i64, _i64, _vp, _vp]
_lib.zo_update_tensor.argtypes = [_vp, _i64, _u64, _i32, _vp, _f32, _vp]
_lib.zo_debug_quant_weight.argtypes = [_vp, _i32, _i32, _i32, _i32, _u64, _i32, _f32, _i32, _vp, _vp, _vp, _vp, _vp]
_lib.zo_debug_quant_act.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
_lib.zo_linear_scratch_bytes.argtypes = [_i32, _i32, _i32, _i32]
_lib.zo_linear_scratch_bytes.restype = _sz
_lib.zo_linear_fakequant.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _u64, _i32, _f32, _vp, _vp]
_lib.zo_linear_fakequant_fused.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _u64, _i32, _f32, _i32, _vp, _vp]
_lib.zo_linear_fused_scratch_bytes.argtypes = [_i32, _i32]
_lib.zo_linear_fused_scratch_bytes.restype = _sz
_lib.zo_linear_frozen_fused_scratch_bytes.argtypes = [_i32, _i32, _i32, _i32]
_lib.zo_linear_frozen_fused_scratch_bytes.restype = _sz
_lib.zo_linear_frozen_int4_fused.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp]
_lib.zo_gemm_nt_swiglu.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _vp]
_lib.zo_gemm_nt.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp]
_lib.zo_gemm_nt_ce.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp]
_lib.zo_gemm_nt_ce_scratch_bytes.argtypes = [_i32, _i32]
_lib.zo_gemm_nt_ce_scratch_bytes.restype = _sz
_lib.zo_profile_begin_mask.argtypes = [_vp, C.c_uint32]
_lib.zo_debug_buffer.argtypes = [_vp, _i32, _i32, C.POINTER(_vp), C.POINTER(_sz)]
_lib.zo_attention_causal.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i64, _i32, _vp, _vp]
_lib.zo_attention_scratch_bytes.argtypes = [_i32, _i32, _i32, _i32, _i32]
_lib.zo_attention_scratch_bytes.restype = _sz
_lib.zo_pack_weight_int4.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.zo_attach_frozen_int4.argtypes = [_vp, _i32, _vp, _vp, _vp, _i32]
_lib.zo_linear_frozen_int4.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp]
_lib.zo_gemm_nt_fused.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp]
_lib.zo_gemm_nt_fused_splitk.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp, _sz, _vp]
_lib.zo_gemm_nt_fused_splitk_static.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp]
_lib.zo_gemm_nt_splitk_static_max_bytes.argtypes = []
_lib.zo_gemm_nt_splitk_static_max_bytes.restype = _sz
_lib.zo_linear_mma_scratch_bytes.argtypes = [_i32, _i32, _i32, _i32, _i32, _i32, C.POINTER(_sz)]
_lib.zo_linear_mma_scratch_bytes.restype = _sz
_lib.zo_linear_fakequant_mma.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _u64, _i32, _f32,
                                         _vp, _vp, _vp]
_lib.zo_linear_frozen_int4_token.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp]
_lib.zo_kv_cache_bytes.argtypes = [C.POINTER(zo_config), _i32]
_lib.zo_kv_cache_bytes.restype = _sz
_lib.zo_prefill.argtypes = [_vp, _vp, _i32, _vp, _i32, _vp]
_lib.zo_decode.argtypes = [_vp, _vp, _i32, _vp, _i32, _vp]
_lib.zo_generate_greedy.argtypes = [_vp, _vp, _i32, _i32, _vp, _i32, _vp, _vp]
_lib.zo_gemm_nt_splitk_ranges.argtypes = [_i32, _i32, _i32, _i32]
_lib.zo_gemm_nt_splitk_ranges.restype = _i32
_lib.zo_gemm_nt_splitk_scratch_bytes.argtypes = [_i32, _i32, _i32, _i32]
_lib.zo_gemm_nt_splitk_scratch_bytes.restype = _sz
_lib.zo_init_learned_params.argtypes = [_vp]
_lib.zo_step_groups.argtypes = [_vp, _vp, _vp, _i32, _i32, _u64, _f32, _f32, _f32, _f32, _vp]
_lib.zo_update_groups.argtypes = [_vp, _u64, _vp, C.POINTER(C.c_float)]
_lib.zo_debug_quant_weight_learned.argtypes = [_vp, _i32, _i32, _i32, _i32, _u64, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]
_lib.zo_debug_smooth_bias.argtypes = [_vp, _i32, _i32, _u64, _i32, _f32, _vp, _vp, _vp, _vp]
_lib.zo_step_multi.argtypes = [_vp, _vp, _vp, _i32, _i32, C.POINTER(_u64), _i32, _f32, _f32, _f32, _f32, _vp]
_lib.zo_update_multi.argtypes = [_vp, C.POINTER(_u64), _i32, _vp, C.POINTER(C.c_float)]
_lib.zo_lr_linear_decay.argtypes = [_f32, _i64, _i64]
_lib.zo_lr_linear_decay.restype = _f32
_lib.zo_update_tensor_f16.argtypes = [_vp, _i64, _u64, _i32, _vp, _f32, _i32, _vp]
_lib.zo_master_bytes.argtypes = [C.POINTER(zo_config)]
_lib.zo_master_bytes.restype = _i64
_lib.zo_debug_routes.argtypes = [_vp]
_lib.zo_debug_routes.restype = C.c_uint32
_lib.zo_profile_begin.argtypes = [_vp]
_lib.zo_profile_end.argtypes = [_vp, C.POINTER(C.c_float), C.POINTER(_i32)]


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(status, where, ctx=None):
    if status != ZO_OK:
        detail = _lib.zo_last_error(ctx).decode() if ctx else ""
        raise ZoError(status, where, detail)


def _tdtype(dtype):
    return torch.bfloat16 if dtype == ACT_BF16 else torch.float32


def make_config(arch, n_layers=0, d_model=0, n_heads=1, d_ffn=0, vocab=0, max_seq=0, w_bits=4, w_group=64,
                a_bits=16, a_sym=0, act_dtype=ACT_FP32, lightweight=0, learn_clip=0, learn_smooth=0, no_fused=0,
                master_dtype=MASTER_F32, master_round=0, mma=0):
    return zo_config(arch, n_layers, d_model, n_heads, d_ffn, vocab, max_seq, w_bits, w_group, a_bits, a_sym,
                     act_dtype, lightweight, learn_clip, learn_smooth, no_fused, master_dtype, master_round, mma)


def zo_master_bytes(cfg):
    return _lib.zo_master_bytes(C.byref(cfg))


def zo_num_params(cfg):
    return _lib.zo_num_params(C.byref(cfg))


def zo_param_numel(cfg, index):
    return _lib.zo_param_numel(C.byref(cfg), index)


def zo_workspace_bytes(cfg, B, S):
    return _lib.zo_workspace_bytes(C.byref(cfg), B, S)


class PackedInt4:
    """Device storage of one frozen, pre-quantized linear (see zo_pack_weight_int4 in the header):
    codes u8 [N][K/2], step f16 [N][K/group], zp i16 [N][K/group]."""

    def __init__(self, codes, step_f16, zp, N, K, group):
        self.codes, self.step_f16, self.zp, self.N, self.K, self.group = codes, step_f16, zp, N, K, group

    def numel(self):
        return self.N * self.K


class Context:
    """Owns nothing on the device except references that keep the caller's tensors alive.
    Entries of `params` are fp32 tensors, or PackedInt4 for frozen linears of a lightweight
    configuration (their `trainable` flag must be false)."""

    def __init__(self, cfg, params, max_B, max_S, trainable=None):
        self.handle = None
        self.cfg = cfg
        self.params = params
        n = len(params)
        arr = (zo_tensor * n)()
        for i, p in enumerate(params):
            tr = 1 if (trainable is None or trainable[i]) else 0
            if isinstance(p, PackedInt4):
                arr[i] = zo_tensor(None, p.numel(), tr, 0)
                continue
            want = torch.float16 if cfg.master_dtype == MASTER_F16 else torch.float32
            assert p.is_cuda and p.dtype == want and p.is_contiguous()
            arr[i] = zo_tensor(p.data_ptr(), p.numel(), tr, 0)
        nbytes = zo_workspace_bytes(cfg, max_B, max_S)
        if nbytes == 0:
            raise ZoError(1, "zo_workspace_bytes")
        dev = next(p for p in params if not isinstance(p, PackedInt4)).device
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.out4 = torch.zeros(4, dtype=torch.float32, device=dev)
        self.handle = _vp()
        _check(_lib.zo_init(C.byref(cfg), arr, n, self.workspace.data_ptr(), nbytes, max_B, max_S, _stream(),
                            C.byref(self.handle)), "zo_init")
        for i, p in enumerate(params):
            if isinstance(p, PackedInt4):
                self.zo_attach_frozen_int4(i, p)

    def zo_attach_frozen_int4(self, index, p):
        _check(_lib.zo_attach_frozen_int4(self.handle, index, p.codes.data_ptr(), p.step_f16.data_ptr(), p.zp.data_ptr(), p.group),
               "zo_attach_frozen_int4", self.handle)

    def close(self):
        if self.handle:
            _lib.zo_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        self.close()

    def zo_forward_quant(self, ids, target, B, S, seed, eps_signed, loss_dev=None):
        loss = loss_dev if loss_dev is not None else torch.zeros(1, dtype=torch.float32, device=ids.device)
        _check(_lib.zo_forward_quant(self.handle, _ptr(ids), _ptr(target), B, S, seed, eps_signed, loss.data_ptr()),
               "zo_forward_quant", self.handle)
        return loss

    # ---- generator on the quantized model (the caller owns the cache, the logits and the token buffers) ----
    def new_kv_cache(self, kv_max_seq):
        nbytes = int(_lib.zo_kv_cache_bytes(C.byref(self.cfg), kv_max_seq))
        if nbytes == 0:
            raise ZoError(1, "zo_kv_cache_bytes")
        return torch.zeros(nbytes, dtype=torch.uint8, device=self.workspace.device)

    def zo_prefill(self, ids, kv, kv_max_seq, logits=None):
        if logits is None:
            logits = torch.empty(self.cfg.vocab, dtype=torch.float32, device=ids.device)
        _check(_lib.zo_prefill(self.handle, ids.data_ptr(), ids.numel(), kv.data_ptr(), kv_max_seq, logits.data_ptr()), "zo_prefill", self.handle)
        return logits

    def zo_decode(self, token, pos, kv, kv_max_seq, logits=None):
        if logits is None:
            logits = torch.empty(self.cfg.vocab, dtype=torch.float32, device=token.device)
        _check(_lib.zo_decode(self.handle, token.data_ptr(), pos, kv.data_ptr(), kv_max_seq, logits.data_ptr()), "zo_decode", self.handle)
        return logits

    def zo_generate_greedy(self, prompt, n_new, kv, kv_max_seq, tokens=None, logits=None):
        if tokens is None:
            tokens = torch.zeros(n_new, dtype=torch.int32, device=prompt.device)
        if logits is None:
            logits = torch.empty(self.cfg.vocab, dtype=torch.float32, device=prompt.device)
        _check(_lib.zo_generate_greedy(self.handle, prompt.data_ptr(), prompt.numel(), n_new, kv.data_ptr(), kv_max_seq, tokens.data_ptr(),
                                       logits.data_ptr()), "zo_generate_greedy", self.handle)
        return tokens, logits

    def zo_step(self, ids, target, B, S, seed, eps, lr, out_dev=None):
        out = out_dev if out_dev is not None else self.out4
        _check(_lib.zo_step(self.handle, _ptr(ids), _ptr(target), B, S, seed, eps, lr, out.data_ptr()), "zo_step", self.handle)
        return out

    def zo_init_learned_params(self):
        _check(_lib.zo_init_learned_params(self.handle), "zo_init_learned_params", self.handle)

    def zo_step_groups(self, ids, target, B, S, seed, eps, lr_model, lr_smooth, lr_clip, out_dev=None):
        out = out_dev if out_dev is not None else torch.zeros(6, dtype=torch.float32, device=ids.device)
        _check(_lib.zo_step_groups(self.handle, _ptr(ids), _ptr(target), B, S, seed, eps, lr_model, lr_smooth, lr_clip,
                                   out.data_ptr()), "zo_step_groups", self.handle)
        return out

    def zo_update_groups(self, seed, coeff_dev=None, coeff_host=None):
        host = None if coeff_host is None else (C.c_float * 3)(*coeff_host)
        _check(_lib.zo_update_groups(self.handle, seed, _ptr(coeff_dev), host), "zo_update_groups", self.handle)

    def zo_step_multi(self, ids, target, B, S, seeds, eps, lr_model, lr_smooth=None, lr_clip=None, out_dev=None):
        q = len(seeds)
        out = out_dev if out_dev is not None else torch.zeros((q, 6), dtype=torch.float32, device=ids.device)
        arr = (_u64 * q)(*seeds)
        _check(_lib.zo_step_multi(self.handle, _ptr(ids), _ptr(target), B, S, arr, q, eps, lr_model,
                                  lr_model if lr_smooth is None else lr_smooth, lr_model if lr_clip is None else lr_clip,
                                  out.data_ptr()), "zo_step_multi", self.handle)
        return out

    def zo_update_multi(self, seeds, coeff_dev=None, coeff_host=None):
        q = len(seeds)
        arr = (_u64 * q)(*seeds)
        host = None if coeff_host is None else (C.c_float * (3 * q))(*[float(v) for row in coeff_host for v in row])
        _check(_lib.zo_update_multi(self.handle, arr, q, _ptr(coeff_dev), host), "zo_update_multi", self.handle)

    def zo_update(self, seed, coeff_dev=None, coeff_host=0.0):
        _check(_lib.zo_update(self.handle, seed, _ptr(coeff_dev), coeff_host), "zo_update", self.handle)

    def zo_debug_routes(self):
        return int(_lib.zo_debug_routes(self.handle))

    def zo_profile_begin(self):
        _check(_lib.zo_profile_begin(self.handle), "zo_profile_begin", self.handle)

    def zo_profile_begin_mask(self, categories):
        """categories: names out of PROF_NAMES whose launches are bracketed."""
        mask = 0
        for name in categories:
            mask |= 1 << PROF_NAMES.index(name)
        _check(_lib.zo_profile_begin_mask(self.handle, mask), "zo_profile_begin_mask", self.handle)

    def zo_profile_end(self):
        """Synchronises; returns {category: (milliseconds, launches)}."""
        ms = (C.c_float * len(PROF_NAMES))()
        n = (_i32 * len(PROF_NAMES))()
        _check(_lib.zo_profile_end(self.handle, ms, n), "zo_profile_end", self.handle)
        return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(PROF_NAMES)}

    def zo_debug_buffer(self, which, branch=0):
        p, n = _vp(), _sz()
        _check(_lib.zo_debug_buffer(self.handle, which, branch, C.byref(p), C.byref(n)), "zo_debug_buffer", self.handle)
        off = p.value - self.workspace.data_ptr()
        return self.workspace[off:off + n.value]


def zo_lr_linear_decay(lr0, t, T):
    return _lib.zo_lr_linear_decay(lr0, t, T)


def zo_probe_mfma_only(workgroups, iters, zero_operands, out=None):
    """Launches the matrix-instruction-only probe on the current stream; returns (out, flop of the launch)."""
    if out is None:
        out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    _check(_lib.zo_probe_mfma_only(out.data_ptr(), workgroups, iters, int(zero_operands), _stream()), "zo_probe_mfma_only")
    return out, 4.0 * 8 * 32768 * iters * workgroups


def zo_debug_philox_u32(seed, tensor_id, nwords, device="cuda"):
    out = torch.empty(nwords, dtype=torch.int32, device=device)
    _check(_lib.zo_debug_philox_u32(seed, tensor_id, nwords, out.data_ptr(), _stream()), "zo_debug_philox_u32")
    return out


def zo_debug_normal(seed, tensor_id, numel, start=0, device="cuda"):
    out = torch.empty(numel, dtype=torch.float32, device=device)
    _check(_lib.zo_debug_normal(seed, tensor_id, start, numel, out.data_ptr(), _stream()), "zo_debug_normal")
    return out


def zo_update_tensor(w, seed, tensor_id, coeff_dev=None, coeff_host=0.0):
    _check(_lib.zo_update_tensor(w.data_ptr(), w.numel(), seed, tensor_id, _ptr(coeff_dev), coeff_host, _stream()),
           "zo_update_tensor")
    return w


def zo_update_tensor_f16(w, seed, tensor_id, coeff_dev=None, coeff_host=0.0, stochastic=False):
    assert w.dtype == torch.float16
    _check(_lib.zo_update_tensor_f16(w.data_ptr(), w.numel(), seed, tensor_id, _ptr(coeff_dev), coeff_host, int(stochastic), _stream()),
           "zo_update_tensor_f16")
    return w


def zo_debug_quant_weight(W, bits, group, seed=0, tensor_id=0, eps_signed=0.0, out_dtype=ACT_FP32, want_codes=True):
    N, K = W.shape
    g = group if group else K
    G = K // g if bits else 0
    dev = W.device
    codes = torch.empty((N, K), dtype=torch.uint8, device=dev) if (bits and want_codes) else None
    step = torch.empty((N, G), dtype=torch.float32, device=dev) if bits else None
    zp = torch.empty((N, G), dtype=torch.int32, device=dev) if bits else None
    what = torch.empty((N, K), dtype=_tdtype(out_dtype), device=dev)
    _check(_lib.zo_debug_quant_weight(W.data_ptr(), N, K, bits, group, seed, tensor_id, eps_signed, out_dtype,
                                      _ptr(codes), _ptr(step), _ptr(zp), what.data_ptr(), _stream()), "zo_debug_quant_weight")
    return dict(codes=codes, step=step, zp=zp, what=what)


def zo_debug_quant_weight_learned(W, bits, group, step, zp, alpha, beta, scale=None, seed=0, tensor_id=0, eps_signed=0.0,
                                  out_dtype=ACT_FP32, want_codes=True):
    N, K = W.shape
    codes = torch.empty((N, K), dtype=torch.uint8, device=W.device) if want_codes else None
    what = torch.empty((N, K), dtype=_tdtype(out_dtype), device=W.device)
    _check(_lib.zo_debug_quant_weight_learned(W.data_ptr(), N, K, bits, group, seed, tensor_id, eps_signed, _ptr(scale),
                                              step.data_ptr(), zp.data_ptr(), alpha.data_ptr(), beta.data_ptr(), out_dtype,
                                              _ptr(codes), what.data_ptr(), _stream()), "zo_debug_quant_weight_learned")
    return dict(codes=codes, what=what)


def zo_debug_smooth_bias(W, delta, bias=None, seed=0, tensor_id=0, eps_signed=0.0):
    N, K = W.shape
    out = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(_lib.zo_debug_smooth_bias(W.data_ptr(), N, K, seed, tensor_id, eps_signed, delta.data_ptr(), _ptr(bias),
                                     out.data_ptr(), _stream()), "zo_debug_smooth_bias")
    return out


def zo_debug_quant_act(X, bits, sym=0, want_codes=True):
    M, K = X.shape
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    dev = X.device
    codes = torch.empty((M, K), dtype=torch.int16, device=dev) if want_codes else None
    step = torch.empty(M, dtype=torch.float32, device=dev)
    zp = torch.empty(M, dtype=torch.int32, device=dev)
    xhat = torch.empty_like(X)
    _check(_lib.zo_debug_quant_act(X.data_ptr(), M, K, bits, sym, dtype, _ptr(codes), step.data_ptr(), zp.data_ptr(),
                                   xhat.data_ptr(), _stream()), "zo_debug_quant_act")
    return dict(codes=codes, step=step, zp=zp, xhat=xhat)


def zo_linear_fakequant(X, W, bias, w_bits, w_group, a_bits, a_sym=0, seed=0, tensor_id=0, eps_signed=0.0, scratch=None):
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    if scratch is None:
        scratch = torch.empty(_lib.zo_linear_scratch_bytes(M, N, K, dtype), dtype=torch.uint8, device=X.device)
    Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    _check(_lib.zo_linear_fakequant(X.data_ptr(), W.data_ptr(), _ptr(bias), Y.data_ptr(), M, N, K, w_bits, w_group,
                                    a_bits, a_sym, dtype, seed, tensor_id, eps_signed, scratch.data_ptr(), _stream()),
           "zo_linear_fakequant")
    return Y


def zo_linear_fakequant_fused(Xp, Xm, W, bias, w_bits, w_group, seed=0, tensor_id=0, eps=0.0, out_f32=False, relayout=False):
    """Both branches (Xm given) or one (Xm None, eps signed); returns (Yp, Ym) with Ym None for one branch.
    relayout: give the call its scratch buffer (activations copied into fragment order first)."""
    M, K = Xp.shape
    scratch = torch.empty(_lib.zo_linear_fused_scratch_bytes(M, K), dtype=torch.uint8, device=Xp.device) if relayout else None
    N = W.shape[0]
    odt = torch.float32 if out_f32 else torch.bfloat16
    Y = torch.empty((2 if Xm is not None else 1, M, N), dtype=odt, device=Xp.device)
    _check(_lib.zo_linear_fakequant_fused(Xp.data_ptr(), _ptr(Xm), W.data_ptr(), _ptr(bias), Y[0].data_ptr(),
                                          Y[1].data_ptr() if Xm is not None else None, M, N, K, w_bits, w_group, seed, tensor_id,
                                          eps, int(out_f32), _ptr(scratch), _stream()), "zo_linear_fakequant_fused")
    return Y[0], (Y[1] if Xm is not None else None)


def zo_pack_weight_int4(W, group):
    N, K = W.shape
    dev = W.device
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    step = torch.empty((N, K // group), dtype=torch.float16, device=dev)
    zp = torch.empty((N, K // group), dtype=torch.int16, device=dev)
    _check(_lib.zo_pack_weight_int4(W.data_ptr(), N, K, group, codes.data_ptr(), step.data_ptr(), zp.data_ptr(), _stream()),
           "zo_pack_weight_int4")
    return PackedInt4(codes, step, zp, N, K, group)


def zo_linear_frozen_int4(X, packed, bias, a_bits, a_sym=0):
    """Returns (Y, w^) -- w^ is the de-quantized operand left in the scratch buffer."""
    M, K = X.shape
    N = packed.N
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    scratch = torch.empty(_lib.zo_linear_scratch_bytes(M, N, K, dtype), dtype=torch.uint8, device=X.device)
    Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    _check(_lib.zo_linear_frozen_int4(X.data_ptr(), packed.codes.data_ptr(), packed.step_f16.data_ptr(), packed.zp.data_ptr(),
                                      _ptr(bias), Y.data_ptr(), M, N, K, packed.group, a_bits, a_sym, dtype,
                                      scratch.data_ptr(), _stream()), "zo_linear_frozen_int4")
    es = X.element_size()
    off = (M * K * es + 255) // 256 * 256
    what = scratch[off:off + N * K * es].view(X.dtype).view(N, K)
    return Y, what


def zo_linear_frozen_int4_fused(Xp, Xm, packed, bias=None, out_f32=False, relayout=False):
    """Both branches (Xm given) or one; returns (Yp, Ym).  relayout: lend the call its scratch buffer (split-K form)."""
    M, K = Xp.shape
    N = packed.N
    odt = torch.float32 if out_f32 else torch.bfloat16
    Y = torch.empty((2 if Xm is not None else 1, M, N), dtype=odt, device=Xp.device)
    scratch = (torch.empty(_lib.zo_linear_frozen_fused_scratch_bytes(M, N, K, packed.group), dtype=torch.uint8, device=Xp.device)
               if relayout else None)
    _check(_lib.zo_linear_frozen_int4_fused(Xp.data_ptr(), _ptr(Xm), packed.codes.data_ptr(), packed.step_f16.data_ptr(),
                                            packed.zp.data_ptr(), _ptr(bias), Y[0].data_ptr(),
                                            Y[1].data_ptr() if Xm is not None else None, M, N, K, packed.group, int(out_f32),
                                            _ptr(scratch), _stream()), "zo_linear_frozen_int4_fused")
    return Y[0], (Y[1] if Xm is not None else None)


def zo_gemm_nt(X, W, Y=None):
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    _check(_lib.zo_gemm_nt(X.data_ptr(), W.data_ptr(), Y.data_ptr(), M, N, K, dtype, _stream()), "zo_gemm_nt")
    return Y


def zo_gemm_nt_swiglu(X, W_interleaved):
    """Y[M][N2/2] = silu(X gate^T) * (X up^T) with the gate / up rows of W interleaved in blocks of 32 channels."""
    M, K = X.shape
    N2 = W_interleaved.shape[0]
    Y = torch.empty((M, N2 // 2), dtype=torch.bfloat16, device=X.device)
    _check(_lib.zo_gemm_nt_swiglu(X.data_ptr(), W_interleaved.data_ptr(), Y.data_ptr(), M, N2, K, _stream()), "zo_gemm_nt_swiglu")
    return Y


def zo_gemm_nt_ce(X, W, ids, S):
    """Row losses [M] of the next-token cross entropy of the logits X W^T (bf16 operands), which are not stored."""
    M, K = X.shape
    N = W.shape[0]
    out = torch.empty(M, dtype=torch.float32, device=X.device)
    scratch = torch.empty(max(_lib.zo_gemm_nt_ce_scratch_bytes(M, N), 16), dtype=torch.uint8, device=X.device)
    _check(_lib.zo_gemm_nt_ce(X.data_ptr(), W.data_ptr(), ids.data_ptr(), out.data_ptr(), M, S, N, K, scratch.data_ptr(), _stream()),
           "zo_gemm_nt_ce")
    return out


def zo_gemm_nt_fused(X, W, bias=None, residual=None, relu=False, Y=None):
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    _check(_lib.zo_gemm_nt_fused(X.data_ptr(), W.data_ptr(), _ptr(bias), _ptr(residual), int(relu), Y.data_ptr(), M, N, K, dtype,
                                 _stream()), "zo_gemm_nt_fused")
    return Y


def zo_gemm_nt_splitk_ranges(M, N, K, dtype=ACT_BF16):
    return int(_lib.zo_gemm_nt_splitk_ranges(M, N, K, dtype))


def zo_gemm_nt_fused_splitk(X, W, bias=None, residual=None, relu=False, Y=None):
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    nbytes = int(_lib.zo_gemm_nt_splitk_scratch_bytes(M, N, K, dtype))
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=X.device)
    _check(_lib.zo_gemm_nt_fused_splitk(X.data_ptr(), W.data_ptr(), _ptr(bias), _ptr(residual), int(relu), Y.data_ptr(), M, N, K, dtype,
                                        scratch.data_ptr(), nbytes, _stream()), "zo_gemm_nt_fused_splitk")
    return Y


def zo_linear_frozen_int4_token(x, packed, bias=None, residual=None, relu=False, out_f32=False):
    y = torch.empty(packed.N, dtype=torch.float32 if out_f32 else torch.bfloat16, device=x.device)
    _check(_lib.zo_linear_frozen_int4_token(x.data_ptr(), packed.codes.data_ptr(), packed.step_f16.data_ptr(), packed.zp.data_ptr(),
                                            _ptr(bias), _ptr(residual), int(relu), y.data_ptr(), packed.N, packed.K, packed.group,
                                            int(out_f32), _stream()), "zo_linear_frozen_int4_token")
    return y


MMA_BF16, MMA_INT8 = 0, 1


def zo_linear_fakequant_mma(X, W, w_bits, w_group, a_bits, seed, tensor_id, eps_signed, mma=MMA_INT8, bias=None, a_sym=False,
                            out_f32=False, parts=False):
    """Returns Y, or (Y, dict of the scratch pieces) with parts=True (integer-code route only).  Raises ZoError(5) if a
    weight operand did not fit a signed byte."""
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    off = (_sz * 8)()
    nbytes = int(_lib.zo_linear_mma_scratch_bytes(M, N, K, w_group, dtype, mma, off))
    if nbytes == 0:
        raise ZoError(2, "zo_linear_mma_scratch_bytes")
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
    flag = torch.zeros(1, dtype=torch.int32, device=X.device)
    Y = torch.empty((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device=X.device)
    _check(_lib.zo_linear_fakequant_mma(X.data_ptr(), W.data_ptr(), _ptr(bias), Y.data_ptr(), M, N, K, w_bits, w_group, a_bits,
                                        int(a_sym), dtype, int(out_f32), mma, seed, tensor_id, eps_signed, scratch.data_ptr(),
                                        flag.data_ptr(), _stream()), "zo_linear_fakequant_mma")
    if int(flag.item()) != 0:
        raise ZoError(5, "zo_linear_fakequant_mma", "a weight operand q - zp does not fit a signed byte")
    if not parts:
        return Y
    G = K // (w_group or K)
    o = list(off)
    piece = lambda i, n, dt: scratch[o[i]:o[i] + n * torch.empty(0, dtype=dt).element_size()].view(dt)
    return Y, dict(x_codes=piece(0, M * K, torch.int8).view(M, K), x_step=piece(1, M, torch.float32), x_off=piece(2, M, torch.float32),
                   w_codes=piece(3, N * K, torch.int8).view(N, K), w_r=piece(5, N, torch.float32),
                   w_rpart=piece(6, N * G, torch.float32).view(N, G))


def zo_gemm_nt_splitk_scratch_bytes(M, N, K, dtype=ACT_BF16):
    return int(_lib.zo_gemm_nt_splitk_scratch_bytes(M, N, K, dtype))


def zo_gemm_nt_splitk_static_max_bytes():
    return int(_lib.zo_gemm_nt_splitk_static_max_bytes())


def zo_gemm_nt_fused_splitk_static(X, W, Y, bias=None, residual=None, relu=False):
    """The caller passes every buffer, Y included: the call itself allocates nothing."""
    M, K = X.shape
    N = W.shape[0]
    dtype = ACT_BF16 if X.dtype == torch.bfloat16 else ACT_FP32
    _check(_lib.zo_gemm_nt_fused_splitk_static(X.data_ptr(), W.data_ptr(), _ptr(bias), _ptr(residual), int(relu), Y.data_ptr(),
                                               M, N, K, dtype, _stream()), "zo_gemm_nt_fused_splitk_static")
    return Y


def zo_attention_causal(qkv, B, S, H, dh):
    """qkv: [B*S, 3*H*dh] fused buffer (q | k | v along the last axis); returns [B*S, H*dh]."""
    dtype = ACT_BF16 if qkv.dtype == torch.bfloat16 else ACT_FP32
    d = H * dh
    out = torch.empty((B * S, d), dtype=qkv.dtype, device=qkv.device)
    es = qkv.element_size()
    base = qkv.data_ptr()
    nscratch = _lib.zo_attention_scratch_bytes(B, S, H, dh, dtype)
    scratch = torch.empty(max(nscratch, 16), dtype=torch.uint8, device=qkv.device)
    _check(_lib.zo_attention_causal(base, base + d * es, base + 2 * d * es, out.data_ptr(), B, S, H, dh, 3 * d, dtype,
                                    scratch.data_ptr(), _stream()), "zo_attention_causal")
    return out
