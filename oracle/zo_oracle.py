"""CPU oracle of the ZeroQAT zeroth-order QAT step -- TEST INFRASTRUCTURE ONLY.

Python face of ``zo_oracle.c`` (element-level definitions, fp32 where an integer
code is decided) plus the model-level forward written with numpy in fp64.  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module.  It imports nothing from the HIP package.

Paper passages followed:
  * uniform quantizer ................ Background, "Quantization" equation
  * group-wise / per-token ........... Appendix "Quantization settings"
  * two-point estimate, q = 1 ........ Eq. (2)
  * ZO-SGD update .................... Eq. (3)
  * lightweight variant .............. Section "Lightweight ZeroQAT" (frozen, pre-quantized
                                       weights; Q and V projections stay trainable)
The transformer around the quantized linears is not defined by the paper; it is the
standard pre-norm decoder named by the benchmark configurations (parity unpinned
beyond the library cross-check in the tests).
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zo_oracle.c")
_LIB = os.path.join(_HERE, "libzo_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-mavx2", "-fopenmp", "-fPIC", "-shared"]


def build(force=False):
    """Compile zo_oracle.c with gcc (no-op if the library is newer than the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = C.CDLL(build())

_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")


def _opt(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


_lib.zo_or_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
_lib.zo_or_philox_words.argtypes = [C.c_uint64, C.c_int32, C.c_int64, _u32p]
_lib.zo_or_word_to_normals.argtypes = [C.c_uint32, _f32p]
_lib.zo_or_z.argtypes = [C.c_uint64, C.c_int32, C.c_int64]
_lib.zo_or_z.restype = C.c_float
_lib.zo_or_normal.argtypes = [C.c_uint64, C.c_int32, C.c_int64, C.c_int64, _f32p]
_lib.zo_or_bf16_round_array.argtypes = [_f32p, C.c_int64, _f32p]
_lib.zo_or_perturb.argtypes = [_f32p, C.c_int64, C.c_uint64, C.c_int32, C.c_float, _f32p]
_lib.zo_or_quant_group.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p]
_lib.zo_or_fakequant_weight.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int32,
                                        C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.zo_or_fakequant_act.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.zo_or_linear.argtypes = [_f32p, _f32p, C.c_void_p, C.c_int, C.c_int, C.c_int, _f64p]
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_i16p = np.ctypeslib.ndpointer(np.int16, flags="C_CONTIGUOUS")
_lib.zo_or_f32_to_f16_bits.argtypes = [C.c_float]
_lib.zo_or_f32_to_f16_bits.restype = C.c_uint16
_lib.zo_or_f16_bits_to_f32.argtypes = [C.c_uint16]
_lib.zo_or_f16_bits_to_f32.restype = C.c_float
_lib.zo_or_quant_group_learned.argtypes = [_f32p, C.c_int, C.c_int, C.c_float, C.c_float, C.c_float, C.c_float,
                                           C.c_void_p, C.c_void_p]
_lib.zo_or_fakequant_weight_learned.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int32, C.c_float,
                                                C.c_void_p, _f32p, _f32p, _f32p, _f32p, C.c_int, C.c_void_p, C.c_void_p]
_lib.zo_or_init_learned.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, _f32p, _f32p, _f32p, _f32p]
_lib.zo_or_smooth_act.argtypes = [_f32p, C.c_int, C.c_int, _f32p, _f32p, _f32p]
_lib.zo_or_pack_int4.argtypes = [_f32p, C.c_int, C.c_int, C.c_int, _u8p, _u16p, _i16p]
_lib.zo_or_dequant_int4.argtypes = [_u8p, _u16p, _i16p, C.c_int, C.c_int, C.c_int, C.c_int, _f32p]
_lib.zo_or_projected_grad.argtypes = [C.c_float, C.c_float, C.c_float]
_lib.zo_or_projected_grad.restype = C.c_float
_lib.zo_or_coeff.argtypes = [C.c_float, C.c_float]
_lib.zo_or_coeff.restype = C.c_float
_lib.zo_or_update.argtypes = [_f32p, C.c_int64, C.c_uint64, C.c_int32, C.c_float]
_lib.zo_or_update_f16.argtypes = [_u16p, C.c_int64, C.c_uint64, C.c_int32, C.c_float, C.c_int]
_lib.zo_or_round_array_f16.argtypes = [_f32p, C.c_int64, C.c_uint64, C.c_int32, C.c_int, _u16p]
_lib.zo_or_round_bits.argtypes = [C.c_uint64, C.c_int32, C.c_int64]
_lib.zo_or_round_bits.restype = C.c_uint32
_lib.zo_or_f32_to_f16_stochastic.argtypes = [C.c_float, C.c_uint32]
_lib.zo_or_f32_to_f16_stochastic.restype = C.c_uint16


# ----------------------------------------------------------------------------
# element-level definitions (thin wrappers over the C file)
# ----------------------------------------------------------------------------
def philox4x32_10(ctr, key):
    out = np.empty(4, np.uint32)
    _lib.zo_or_philox4x32_10(np.asarray(ctr, np.uint32), np.asarray(key, np.uint32), out)
    return out


def philox_words(seed, tensor_id, nwords):
    out = np.empty(nwords, np.uint32)
    _lib.zo_or_philox_words(seed, tensor_id, nwords, out)
    return out


def word_to_normals(word):
    out = np.empty(2, np.float32)
    _lib.zo_or_word_to_normals(int(word), out)
    return out


def z_at(seed, tensor_id, i):
    return np.float32(_lib.zo_or_z(seed, tensor_id, i))


def normal(seed, tensor_id, n, start=0):
    out = np.empty(n, np.float32)
    _lib.zo_or_normal(seed, tensor_id, start, n, out)
    return out


def bf16_round(x):
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty_like(x)
    _lib.zo_or_bf16_round_array(x.reshape(-1), x.size, out.reshape(-1))
    return out


def perturb(w, seed, tensor_id, eps_signed):
    """theta' = fma(eps_signed, z, theta) in fp32 (argument of Q in Eq. 2)."""
    w = np.ascontiguousarray(w, np.float32)
    out = np.empty_like(w)
    _lib.zo_or_perturb(w.reshape(-1), w.size, seed, tensor_id, eps_signed, out.reshape(-1))
    return out


def quant_group(x, bits, sym=False):
    """One group through the uniform quantizer: (step, zero_point, codes, dequantized)."""
    x = np.ascontiguousarray(x, np.float32).reshape(-1)
    step = np.empty(1, np.float32)
    zp = np.empty(1, np.int32)
    codes = np.empty(x.size, np.int32)
    xhat = np.empty(x.size, np.float32)
    _lib.zo_or_quant_group(x, x.size, bits, int(sym), _opt(step), _opt(zp), _opt(codes), _opt(xhat))
    return step[0], int(zp[0]), codes, xhat


def fakequant_weight(W, bits, group, seed=0, tensor_id=0, eps_signed=0.0, round_bf16=False, want_codes=True):
    """Q(W + eps_signed*z) per group of `group` consecutive in-features (Eq. 2's Q for a linear).

    Returns dict(codes[N,K] int32, step[N,K/group], zp[N,K/group] int32, what[N,K] fp32)."""
    W = np.ascontiguousarray(W, np.float32)
    N, K = W.shape
    if bits:
        if group == 0:
            group = K
        assert K % group == 0
    G = K // group if bits else 0
    codes = np.empty((N, K), np.int32) if (bits and want_codes) else None
    step = np.empty((N, G), np.float32) if bits else None
    zp = np.empty((N, G), np.int32) if bits else None
    what = np.empty((N, K), np.float32)
    _lib.zo_or_fakequant_weight(W, N, K, bits, group, seed, tensor_id, eps_signed, int(round_bf16),
                                _opt(codes), _opt(step), _opt(zp), _opt(what))
    return dict(codes=codes, step=step, zp=zp, what=what)


def fakequant_act(X, bits, sym=False, round_bf16=False, want_codes=True):
    """Per-token quantizer: every row of X[M,K] is one group."""
    X = np.ascontiguousarray(X, np.float32)
    M, K = X.shape
    q = bits < 16
    codes = np.empty((M, K), np.int32) if (q and want_codes) else None
    step = np.empty(M, np.float32) if q else None
    zp = np.empty(M, np.int32) if q else None
    xhat = np.empty((M, K), np.float32)
    _lib.zo_or_fakequant_act(X, M, K, bits, int(sym), int(round_bf16), _opt(codes), _opt(step), _opt(zp), _opt(xhat))
    return dict(codes=codes, step=step, zp=zp, xhat=xhat)


def quant_group_learned(x, bits, step, zp, alpha, beta):
    """One group through the adaptive weight quantizer of Eq. 5: (codes, dequantized)."""
    x = np.ascontiguousarray(x, np.float32).reshape(-1)
    codes = np.empty(x.size, np.int32)
    xhat = np.empty(x.size, np.float32)
    _lib.zo_or_quant_group_learned(x, x.size, bits, step, zp, alpha, beta, _opt(codes), _opt(xhat))
    return codes, xhat


def fakequant_weight_learned(W, bits, group, step, zp, alpha, beta, scale=None, seed=0, tensor_id=0, eps_signed=0.0,
                             round_bf16=False, want_codes=True):
    """Eq. 5 on scale (.) (W + eps_signed*u) with the given (already perturbed) per-group parameters."""
    W = np.ascontiguousarray(W, np.float32)
    N, K = W.shape
    group = group or K
    f = lambda a: np.ascontiguousarray(a, np.float32).reshape(N, K // group)
    sc = None if scale is None else np.ascontiguousarray(scale, np.float32)
    codes = np.empty((N, K), np.int32) if want_codes else None
    what = np.empty((N, K), np.float32)
    _lib.zo_or_fakequant_weight_learned(W, N, K, bits, group, seed, tensor_id, eps_signed, _opt(sc), f(step), f(zp),
                                        f(alpha), f(beta), int(round_bf16), _opt(codes), _opt(what))
    return dict(codes=codes, what=what)


def init_learned(W, bits, group, scale=None):
    """Initial (step, zp, alpha, beta) per group: the default asymmetric scheme on scale (.) W; alpha 0, beta 1."""
    W = np.ascontiguousarray(W, np.float32)
    N, K = W.shape
    group = group or K
    sc = None if scale is None else np.ascontiguousarray(scale, np.float32)
    out = [np.empty((N, K // group), np.float32) for _ in range(4)]
    _lib.zo_or_init_learned(W, N, K, bits, group, _opt(sc), *out)
    return out


def smooth_act(X, delta, inv_s):
    X = np.ascontiguousarray(X, np.float32)
    out = np.empty_like(X)
    _lib.zo_or_smooth_act(X, X.shape[0], X.shape[1], np.ascontiguousarray(delta, np.float32),
                          np.ascontiguousarray(inv_s, np.float32), out)
    return out


def f32_to_f16_bits(v):
    return int(_lib.zo_or_f32_to_f16_bits(float(np.float32(v))))


def f16_bits_to_f32(h):
    return np.float32(_lib.zo_or_f16_bits_to_f32(int(h)))


class PackedInt4:
    """A frozen, pre-quantized weight matrix of the lightweight variant: 4-bit codes two per byte
    (low nibble = even in-feature), one binary16 step and one int16 zero point per group."""

    def __init__(self, codes, step_f16, zp, N, K, group):
        self.codes, self.step_f16, self.zp, self.N, self.K, self.group = codes, step_f16, zp, N, K, group


def pack_int4(W, group):
    """Pre-quantize W[N,K] with the asymmetric 4-bit group quantizer (no perturbation)."""
    W = np.ascontiguousarray(W, np.float32)
    N, K = W.shape
    assert K % group == 0 and group % 2 == 0
    codes = np.empty((N, K // 2), np.uint8)
    step = np.empty((N, K // group), np.uint16)
    zp = np.empty((N, K // group), np.int16)
    _lib.zo_or_pack_int4(W, N, K, group, codes, step, zp)
    return PackedInt4(codes, step, zp, N, K, group)


def dequant_int4(p, round_bf16=False):
    """w^ = (code - zp) * step of a packed matrix, fp32 (optionally rounded to bf16)."""
    what = np.empty((p.N, p.K), np.float32)
    _lib.zo_or_dequant_int4(p.codes, p.step_f16, p.zp, p.N, p.K, p.group, int(round_bf16), what)
    return what


def linear(xhat, what, bias=None):
    """y = x^ w^T + bias with fp64 accumulation (plain triple loop in C)."""
    xhat = np.ascontiguousarray(xhat, np.float32)
    what = np.ascontiguousarray(what, np.float32)
    M, K = xhat.shape
    N = what.shape[0]
    y = np.empty((M, N), np.float64)
    b = None if bias is None else np.ascontiguousarray(bias, np.float32)
    _lib.zo_or_linear(xhat, what, _opt(b), M, N, K, y)
    return y


def projected_grad(loss_plus, loss_minus, eps):
    return np.float32(_lib.zo_or_projected_grad(loss_plus, loss_minus, eps))


def coeff(lr, g):
    return np.float32(_lib.zo_or_coeff(lr, g))


def update(w, seed, tensor_id, c, stochastic=False):
    """In place: w <- fma(-c, z, w) (Eq. 3).  Masters kept in binary16 (dtype float16) are rounded once
    after the fp32 fma: to nearest even, or stochastically."""
    assert w.flags.c_contiguous
    if w.dtype == np.float16:
        _lib.zo_or_update_f16(w.reshape(-1).view(np.uint16), w.size, seed, tensor_id, c, int(stochastic))
        return w
    assert w.dtype == np.float32
    _lib.zo_or_update(w.reshape(-1), w.size, seed, tensor_id, c)
    return w


def update_multi(w, seeds, tensor_id, cs, stochastic=False):
    """In place: the q rank-one terms of a q-direction step in seed order, one fp32 fma each.  binary16 masters are
    widened once, take all q terms in fp32 and are rounded once at the end (the stochastic rounding draws from the
    rounding stream of the first seed)."""
    if w.dtype == np.float16:
        x = w.astype(np.float32)
        for s, c in zip(seeds, cs):
            update(x, s, tensor_id, c)
        _lib.zo_or_round_array_f16(x.reshape(-1), x.size, seeds[0], tensor_id, int(stochastic), w.reshape(-1).view(np.uint16))
        return w
    for s, c in zip(seeds, cs):
        update(w, s, tensor_id, c)
    return w


def round_bits(seed, tensor_id, i):
    """The 24-bit uniform integer that decides the stochastic rounding of element i."""
    return int(_lib.zo_or_round_bits(seed, tensor_id, i))


def f32_to_f16_stochastic(x, r):
    """binary16 bits of x rounded stochastically with the 24-bit integer r."""
    return int(_lib.zo_or_f32_to_f16_stochastic(float(np.float32(x)), int(r)))


# ----------------------------------------------------------------------------
# model-level forward (numpy, fp64 inside every operation)
# ----------------------------------------------------------------------------
ARCH_LINEAR, ARCH_LLAMA, ARCH_OPT = 0, 1, 2


class Config:
    """Mirror of the library's configuration record (field meaning identical)."""

    def __init__(self, arch, n_layers=0, d_model=0, n_heads=1, d_ffn=0, vocab=0, max_seq=0,
                 w_bits=4, w_group=64, a_bits=16, a_sym=0, act_dtype=0, lightweight=0, learn_clip=0, learn_smooth=0, mma=0):
        self.arch, self.n_layers, self.d_model, self.n_heads = arch, n_layers, d_model, n_heads
        self.d_ffn, self.vocab, self.max_seq = d_ffn, vocab, max_seq
        self.w_bits, self.w_group, self.a_bits, self.a_sym = w_bits, w_group, a_bits, a_sym
        self.act_dtype, self.lightweight = act_dtype, lightweight
        # learnable quantizer parameters (Eq. 5) / channel-wise smoothing (Eq. 4) as ZO-trained tensors
        self.learn_clip, self.learn_smooth = learn_clip, learn_smooth
        # mma = 1: a quantized linear with weight and activation codes contracts the integer codes themselves, so its
        # operands are the quantizer's outputs (code - zp) * step as they are -- NOT rounded to bf16 first, whatever the
        # storage type of activations (the rounding of GEMM operands in bf16 mode is a property of the bf16 contraction,
        # not of the quantizer of the Background section).  Stored activations are still rounded to act_dtype.
        self.mma = mma


GROUP_MODEL, GROUP_SMOOTH, GROUP_CLIP = 0, 1, 2      # learning-rate groups (Appendix, hyperparameter table)


def param_shapes(cfg):
    """Ordered (name, shape, quantized?) of the trainable tensors; index = tensor id.

    The model's own tensors come first; then, for every quantized linear in that order, the
    tensors of its adaptive quantizer (Eq. 5: step, zero point, alpha, beta, one value per group)
    when cfg.learn_clip, and of the smoothing of its input (Eq. 4: s and delta, one value per input
    feature) when cfg.learn_smooth.  Linears that read the same activation (q/k/v; gate/up) share
    one smoothing pair, listed with the first of them: one activation has one quantized form."""
    base = _base_param_shapes(cfg)
    out = list(base)
    for name, (N, K), q in [b for b in base if b[2]]:
        G = K // (cfg.w_group or K)
        if getattr(cfg, "learn_clip", 0):
            out += [(name + sfx, (N, G), False) for sfx in (".q_step", ".q_zp", ".q_alpha", ".q_beta")]
        if getattr(cfg, "learn_smooth", 0) and smooth_owner(name) == name:
            out += [(name + ".sm_s", (K,), False), (name + ".sm_delta", (K,), False)]
    return out


def smooth_owner(name):
    """Name of the linear that carries the smoothing pair of `name`'s input activation."""
    head, _, last = name.rpartition(".")
    owner = {"wk": "wq", "wv": "wq", "w_up": "w_gate"}.get(last, last)
    return (head + "." if head else "") + owner


def param_groups(cfg):
    """Learning-rate group of every tensor, in param_shapes order."""
    g = []
    for name, _, _ in param_shapes(cfg):
        last = name.split(".")[-1]
        g.append(GROUP_CLIP if last.startswith("q_") else GROUP_SMOOTH if last.startswith("sm_") else GROUP_MODEL)
    return g


def init_learned_params(cfg, params):
    """Fill the quantizer / smoothing tensors of `params` (a list in param_shapes order) in place:
    s = 1, delta = 0 (identity smoothing), then Eq. 5's parameters from the default scheme."""
    index = {name: i for i, (name, _, _) in enumerate(param_shapes(cfg))}
    for name, shape, q in _base_param_shapes(cfg):
        if not q:
            continue
        scale = None
        if cfg.learn_smooth:
            own = smooth_owner(name)
            params[index[own + ".sm_s"]][...] = 1.0
            params[index[own + ".sm_delta"]][...] = 0.0
            scale = params[index[own + ".sm_s"]]
        if cfg.learn_clip:
            vals = init_learned(params[index[name]], cfg.w_bits, cfg.w_group, scale)
            for sfx, v in zip((".q_step", ".q_zp", ".q_alpha", ".q_beta"), vals):
                params[index[name + sfx]][...] = v
    return params


def _base_param_shapes(cfg):
    d, f, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    if cfg.arch == ARCH_LINEAR:
        return [("w", (f, d), True)]
    out = [("tok_emb", (V, d), False)]
    if cfg.arch == ARCH_OPT:
        out.append(("pos_emb", (cfg.max_seq, d), False))
    for l in range(cfg.n_layers):
        p = "l%d." % l
        if cfg.arch == ARCH_LLAMA:
            out += [(p + "attn_norm", (d,), False), (p + "wq", (d, d), True), (p + "wk", (d, d), True),
                    (p + "wv", (d, d), True), (p + "wo", (d, d), True), (p + "ffn_norm", (d,), False),
                    (p + "w_gate", (f, d), True), (p + "w_up", (f, d), True), (p + "w_down", (d, f), True)]
        else:
            out += [(p + "ln1_g", (d,), False), (p + "ln1_b", (d,), False),
                    (p + "wq", (d, d), True), (p + "bq", (d,), False), (p + "wk", (d, d), True), (p + "bk", (d,), False),
                    (p + "wv", (d, d), True), (p + "bv", (d,), False), (p + "wo", (d, d), True), (p + "bo", (d,), False),
                    (p + "ln2_g", (d,), False), (p + "ln2_b", (d,), False),
                    (p + "fc1", (f, d), True), (p + "b1", (f,), False), (p + "fc2", (d, f), True), (p + "b2", (d,), False)]
    if cfg.arch == ARCH_LLAMA:
        out += [("final_norm", (d,), False), ("lm_head", (V, d), False)]
    else:
        out += [("final_ln_g", (d,), False), ("final_ln_b", (d,), False), ("lm_head", (V, d), False)]
    return out


def _operand_bf16(cfg):
    """Are the operands of a quantized linear rounded to bf16 before they are multiplied?"""
    return cfg.act_dtype == 1 and not (cfg.mma == 1 and cfg.w_bits > 0 and cfg.a_bits <= 8)


def _rt(cfg, a):
    """Round to the storage type of activations (bf16 in bf16 mode, fp32 otherwise)."""
    a32 = np.asarray(a, np.float64).astype(np.float32)
    return bf16_round(a32) if cfg.act_dtype == 1 else a32


class _Params:
    """Perturbed view of the parameter list: theta'_i = fma(eps_signed, z, theta_i)."""

    def __init__(self, cfg, params, seed, eps_signed, trainable=None):
        self.cfg, self.params, self.seed, self.eps = cfg, params, seed, np.float32(eps_signed)
        self.index = {name: i for i, (name, _, _) in enumerate(param_shapes(cfg))}
        self.trainable = trainable

    def _eps_for(self, i):
        if self.trainable is not None and not self.trainable[i]:
            return np.float32(0.0)
        return self.eps

    def plain(self, name):
        """Perturbed, un-quantized fp32 tensor (norm gains, biases, embeddings)."""
        i = self.index[name]
        return perturb(self.params[i], self.seed, i, self._eps_for(i))

    def lm_head(self, name):
        """Perturbed un-quantized matrix, rounded to the GEMM operand type."""
        i = self.index[name]
        return fakequant_weight(self.params[i], 0, 0, self.seed, i, self._eps_for(i),
                                round_bf16=(self.cfg.act_dtype == 1), want_codes=False)["what"]

    def qweight(self, name):
        """Q(W + eps z) of a quantized linear, de-quantized, in the GEMM operand type."""
        i = self.index[name]
        cfg = self.cfg
        if isinstance(self.params[i], PackedInt4):     # frozen and pre-quantized: used as stored
            assert self.trainable is not None and not self.trainable[i]
            return dequant_int4(self.params[i], round_bf16=_operand_bf16(cfg))
        scale = self.plain(smooth_owner(name) + ".sm_s") if cfg.learn_smooth else None
        if cfg.learn_clip:
            qp = [self.plain(name + sfx) for sfx in (".q_step", ".q_zp", ".q_alpha", ".q_beta")]
            return fakequant_weight_learned(self.params[i], cfg.w_bits, cfg.w_group, *qp, scale=scale, seed=self.seed,
                                            tensor_id=i, eps_signed=self._eps_for(i),
                                            round_bf16=_operand_bf16(cfg), want_codes=False)["what"]
        if scale is not None:
            # smoothing with the dynamic quantizer: min/max of every group of s (.) (W + eps u)
            wb = (perturb(self.params[i], self.seed, i, self._eps_for(i)) * scale[None, :]).astype(np.float32)
            return fakequant_weight(wb, cfg.w_bits, cfg.w_group, round_bf16=_operand_bf16(cfg), want_codes=False)["what"]
        return fakequant_weight(self.params[i], cfg.w_bits, cfg.w_group, self.seed, i, self._eps_for(i),
                                round_bf16=_operand_bf16(cfg), want_codes=False)["what"]

    def smooth(self, name):
        """Activation side and bias term of Eq. 4 for linear `name`: (delta', 1/s', delta' W'^T) or None."""
        if not self.cfg.learn_smooth:
            return None
        i = self.index[name]
        s = self.plain(smooth_owner(name) + ".sm_s")
        delta = self.plain(smooth_owner(name) + ".sm_delta")
        inv_s = (np.float32(1.0) / s).astype(np.float32)
        wp = perturb(self.params[i], self.seed, i, self._eps_for(i))
        shift = wp.astype(np.float64) @ delta.astype(np.float64)
        return delta, inv_s, shift


def _tie_margin(x, step):
    """Per row: distance (in code units) of the closest element to a rounding boundary of
    round(x / step).  A test uses it to know where a last-bit difference in x may flip a code."""
    t = np.asarray(x, np.float32) * (np.float32(1.0) / step.astype(np.float32))[:, None]
    return np.abs(np.abs(t - np.floor(t)) - np.float32(0.5)).min(axis=1)


def _qlinear(cfg, x, what, bias=None, residual=None, relu=False, tie_log=None, smooth=None):
    """Quantized linear: per-token Q_A on the stored input, then x^ w^T (+bias)(+relu)(+residual).
    With smoothing (Eq. 4) the quantizer sees (x - delta) / s and the bias gains delta W^T."""
    if smooth is not None:
        delta, inv_s, shift = smooth
        x = smooth_act(x, delta, inv_s)
        bias = shift if bias is None else bias.astype(np.float64) + shift
    qa = fakequant_act(x, cfg.a_bits, cfg.a_sym, round_bf16=_operand_bf16(cfg), want_codes=False)
    xq = qa["xhat"]
    if tie_log is not None and cfg.a_bits < 16:
        tie_log.append(_tie_margin(x, qa["step"]))
    y = xq.astype(np.float64) @ what.astype(np.float64).T
    if bias is not None:
        y = y + bias.astype(np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    if residual is not None:
        y = y + residual.astype(np.float64)
    return _rt(cfg, y)


def _rmsnorm(x, g, eps=1e-5):
    x = x.astype(np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g.astype(np.float64)


def _layernorm(x, g, b, eps=1e-5):
    x = x.astype(np.float64)
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g.astype(np.float64) + b.astype(np.float64)


def rope_table(S, dh, theta=10000.0):
    """cos/sin of pos * theta^(-2i/dh), i < dh/2, rounded to fp32 (a constant table of the model)."""
    i = np.arange(dh // 2, dtype=np.float64)
    ang = np.arange(S, dtype=np.float64)[:, None] * theta ** (-2.0 * i / dh)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def _rope(x, B, S, H, dh):
    """Rotate pairs (i, i + dh/2) of every head by the position angle."""
    cos, sin = rope_table(S, dh)
    x = x.astype(np.float64).reshape(B, S, H, dh)
    x1, x2 = x[..., : dh // 2], x[..., dh // 2:]
    c = cos.astype(np.float64)[None, :, None, :]
    s = sin.astype(np.float64)[None, :, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], -1).reshape(B * S, H * dh)


def _attention(q, k, v, B, S, H, dh):
    """Causal softmax attention, scale 1/sqrt(dh), fp64."""
    q = q.astype(np.float64).reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    k = k.astype(np.float64).reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    v = v.astype(np.float64).reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    s = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    mask = np.triu(np.ones((S, S), bool), 1)
    s = np.where(mask, -np.inf, s)
    s = s - s.max(-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(-1, keepdims=True)
    return (p @ v).transpose(0, 2, 1, 3).reshape(B * S, H * dh)


def cross_entropy(logits, ids, B, S):
    """Mean over the B*(S-1) next-token positions of logsumexp(logits) - logits[target]."""
    V = logits.shape[-1]
    lg = logits.astype(np.float64).reshape(B, S, V)[:, :-1, :]
    tgt = np.asarray(ids).reshape(B, S)[:, 1:]
    mx = lg.max(-1, keepdims=True)
    lse = np.log(np.exp(lg - mx).sum(-1)) + mx[..., 0]
    picked = np.take_along_axis(lg, tgt[..., None], -1)[..., 0]
    return np.float32((lse - picked).mean())


def forward(cfg, params, ids=None, x=None, target=None, seed=0, eps_signed=0.0, trainable=None, trace=None,
            tie_log=None):
    """One quantized forward at W + eps_signed * z; returns the fp32 loss.

    arch 0: x[M,K] fp32 input, target[M,N]; loss = mean squared error.
    arch 1/2: ids[B,S]; loss = next-token cross entropy.
    `trace`, if a dict, receives the stored activations by name; `tie_log`, if a list, receives
    for every activation-quantizer call the per-row margin to the nearest rounding boundary."""
    P = _Params(cfg, params, seed, eps_signed, trainable)

    def keep(name, val):
        if trace is not None:
            trace[name] = val
        return val

    if cfg.arch == ARCH_LINEAR:
        y = _qlinear(cfg, _rt(cfg, x), P.qweight("w"), tie_log=tie_log, smooth=P.smooth("w"))
        keep("y", y)
        return np.float32(np.mean((y.astype(np.float64) - np.asarray(target, np.float64)) ** 2))

    B, S = np.asarray(ids).shape
    d, H = cfg.d_model, cfg.n_heads
    dh = d // H
    flat = np.asarray(ids).reshape(-1)
    emb = P.plain("tok_emb")
    if cfg.arch == ARCH_OPT:
        pos = P.plain("pos_emb")
        xres = _rt(cfg, emb[flat].astype(np.float64) + np.tile(pos[:S], (B, 1)).astype(np.float64))
    else:
        xres = _rt(cfg, emb[flat])
    keep("x0", xres)
    for l in range(cfg.n_layers):
        p = "l%d." % l
        if cfg.arch == ARCH_LLAMA:
            h = _rt(cfg, _rmsnorm(xres, P.plain(p + "attn_norm")))
            q = _qlinear(cfg, h, P.qweight(p + "wq"), tie_log=tie_log, smooth=P.smooth(p + "wq"))
            k = _qlinear(cfg, h, P.qweight(p + "wk"), tie_log=tie_log, smooth=P.smooth(p + "wk"))
            v = _qlinear(cfg, h, P.qweight(p + "wv"), tie_log=tie_log, smooth=P.smooth(p + "wv"))
            q = _rt(cfg, _rope(q, B, S, H, dh))
            k = _rt(cfg, _rope(k, B, S, H, dh))
            keep(p + "qkv", np.concatenate([q, k, v], axis=1))
            a = keep(p + "attn", _rt(cfg, _attention(q, k, v, B, S, H, dh)))
            xres = _qlinear(cfg, a, P.qweight(p + "wo"), residual=xres, tie_log=tie_log, smooth=P.smooth(p + "wo"))
            keep(p + "attn_out", xres)
            h = _rt(cfg, _rmsnorm(xres, P.plain(p + "ffn_norm")))
            gate = _qlinear(cfg, h, P.qweight(p + "w_gate"), tie_log=tie_log, smooth=P.smooth(p + "w_gate"))
            up = _qlinear(cfg, h, P.qweight(p + "w_up"), tie_log=tie_log, smooth=P.smooth(p + "w_up"))
            g64 = gate.astype(np.float64)
            act = _rt(cfg, g64 / (1.0 + np.exp(-g64)) * up.astype(np.float64))
            xres = _qlinear(cfg, act, P.qweight(p + "w_down"), residual=xres, tie_log=tie_log, smooth=P.smooth(p + "w_down"))
        else:
            h = _rt(cfg, _layernorm(xres, P.plain(p + "ln1_g"), P.plain(p + "ln1_b")))
            q = _qlinear(cfg, h, P.qweight(p + "wq"), P.plain(p + "bq"), tie_log=tie_log, smooth=P.smooth(p + "wq"))
            k = _qlinear(cfg, h, P.qweight(p + "wk"), P.plain(p + "bk"), tie_log=tie_log, smooth=P.smooth(p + "wk"))
            v = _qlinear(cfg, h, P.qweight(p + "wv"), P.plain(p + "bv"), tie_log=tie_log, smooth=P.smooth(p + "wv"))
            keep(p + "qkv", np.concatenate([q, k, v], axis=1))
            a = keep(p + "attn", _rt(cfg, _attention(q, k, v, B, S, H, dh)))
            xres = _qlinear(cfg, a, P.qweight(p + "wo"), P.plain(p + "bo"), residual=xres, tie_log=tie_log, smooth=P.smooth(p + "wo"))
            keep(p + "attn_out", xres)
            h = _rt(cfg, _layernorm(xres, P.plain(p + "ln2_g"), P.plain(p + "ln2_b")))
            f = _qlinear(cfg, h, P.qweight(p + "fc1"), P.plain(p + "b1"), relu=True, tie_log=tie_log, smooth=P.smooth(p + "fc1"))
            xres = _qlinear(cfg, f, P.qweight(p + "fc2"), P.plain(p + "b2"), residual=xres, tie_log=tie_log, smooth=P.smooth(p + "fc2"))
        keep(p + "out", xres)
    if cfg.arch == ARCH_LLAMA:
        hf = _rt(cfg, _rmsnorm(xres, P.plain("final_norm")))
    else:
        hf = _rt(cfg, _layernorm(xres, P.plain("final_ln_g"), P.plain("final_ln_b")))
    keep("final", hf)
    logits = hf.astype(np.float64) @ P.lm_head("lm_head").astype(np.float64).T
    keep("logits", logits)
    return cross_entropy(logits, ids, B, S)


# ---- inference on the trained (quantized) model: prompt pass + token-by-token decoding with a key / value cache ----
# The efficiency section's on-device table runs the quantized model as a generator (prompt of a few hundred tokens,
# then one token at a time).  The computation is the quantized forward above at eps = 0 restricted to what a generator
# needs: every layer keeps the keys (after the rotary embedding) and values of the positions seen so far, as stored
# activations; a new token's query attends to all of them.  Per-token activation quantizers make every row independent of
# the others, so a cached step computes exactly what the full forward computes at that position.

def _rope_rows(x, pos, H, dh):
    """Rotate pairs (i, i + dh/2) of every head of row r by the angle of position pos[r]."""
    cos, sin = rope_table(int(np.max(pos)) + 1, dh)
    T = x.shape[0]
    x = x.astype(np.float64).reshape(T, H, dh)
    x1, x2 = x[..., : dh // 2], x[..., dh // 2:]
    c = cos.astype(np.float64)[pos][:, None, :]
    s_ = sin.astype(np.float64)[pos][:, None, :]
    return np.concatenate([x1 * c - x2 * s_, x2 * c + x1 * s_], -1).reshape(T, H * dh)


def _attend_rows(q, K, V, pos, H, dh):
    """Row r (position pos[r]) attends to cache rows 0 .. pos[r]; plain loops over rows and heads, fp64."""
    T = q.shape[0]
    out = np.zeros((T, H * dh), np.float64)
    for r in range(T):
        n = int(pos[r]) + 1
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            sc = K[:n, sl].astype(np.float64) @ q[r, sl].astype(np.float64) / np.sqrt(dh)
            sc = np.exp(sc - sc.max())
            out[r, sl] = (sc / sc.sum()) @ V[:n, sl].astype(np.float64)
    return out


def _infer_rows(cfg, params, tokens, pos, kv, trainable):
    """Rows for `tokens` at positions `pos` (consecutive, starting at the cache length); extends kv; returns the final
    hidden states (stored type) of those rows."""
    P = _Params(cfg, params, 0, 0.0, trainable)
    d, H = cfg.d_model, cfg.n_heads
    dh = d // H
    tokens = np.asarray(tokens).reshape(-1)
    pos = np.asarray(pos).reshape(-1)
    emb = P.plain("tok_emb")
    if cfg.arch == ARCH_OPT:
        xres = _rt(cfg, emb[tokens].astype(np.float64) + P.plain("pos_emb")[pos].astype(np.float64))
    else:
        xres = _rt(cfg, emb[tokens])
    for l in range(cfg.n_layers):
        p = "l%d." % l
        llama = cfg.arch == ARCH_LLAMA
        if llama:
            h = _rt(cfg, _rmsnorm(xres, P.plain(p + "attn_norm")))
            bq = bk = bv = bo = None
        else:
            h = _rt(cfg, _layernorm(xres, P.plain(p + "ln1_g"), P.plain(p + "ln1_b")))
            bq, bk, bv, bo = (P.plain(p + n) for n in ("bq", "bk", "bv", "bo"))
        q = _qlinear(cfg, h, P.qweight(p + "wq"), bq)
        k = _qlinear(cfg, h, P.qweight(p + "wk"), bk)
        v = _qlinear(cfg, h, P.qweight(p + "wv"), bv)
        if llama:
            q = _rt(cfg, _rope_rows(q, pos, H, dh))
            k = _rt(cfg, _rope_rows(k, pos, H, dh))
        K = k if kv[l][0] is None else np.concatenate([kv[l][0], k], 0)
        V = v if kv[l][1] is None else np.concatenate([kv[l][1], v], 0)
        kv[l] = (K, V)
        a = _rt(cfg, _attend_rows(q, K, V, pos, H, dh))
        xres = _qlinear(cfg, a, P.qweight(p + "wo"), bo, residual=xres)
        if llama:
            h = _rt(cfg, _rmsnorm(xres, P.plain(p + "ffn_norm")))
            gate = _qlinear(cfg, h, P.qweight(p + "w_gate"))
            up = _qlinear(cfg, h, P.qweight(p + "w_up"))
            g64 = gate.astype(np.float64)
            act = _rt(cfg, g64 / (1.0 + np.exp(-g64)) * up.astype(np.float64))
            xres = _qlinear(cfg, act, P.qweight(p + "w_down"), residual=xres)
        else:
            h = _rt(cfg, _layernorm(xres, P.plain(p + "ln2_g"), P.plain(p + "ln2_b")))
            f = _qlinear(cfg, h, P.qweight(p + "fc1"), P.plain(p + "b1"), relu=True)
            xres = _qlinear(cfg, f, P.qweight(p + "fc2"), P.plain(p + "b2"), residual=xres)
    if cfg.arch == ARCH_LLAMA:
        return _rt(cfg, _rmsnorm(xres, P.plain("final_norm"))), P
    return _rt(cfg, _layernorm(xres, P.plain("final_ln_g"), P.plain("final_ln_b"))), P


def new_kv(cfg):
    return [(None, None) for _ in range(cfg.n_layers)]


def infer_prefill(cfg, params, prompt, kv, trainable=None):
    """Prompt pass of one sequence: fills kv (per layer: keys after the rotary embedding and values of every position, in
    the activation storage type) and returns the logits (fp64 [V]) of the LAST position -- the distribution of the first
    generated token."""
    assert not (cfg.learn_clip or cfg.learn_smooth)
    prompt = np.asarray(prompt).reshape(-1)
    hf, P = _infer_rows(cfg, params, prompt, np.arange(prompt.size), kv, trainable)
    return hf[-1].astype(np.float64) @ P.lm_head("lm_head").astype(np.float64).T


def infer_decode(cfg, params, token, kv, trainable=None):
    """One more token: its position is the current cache length; returns the logits (fp64 [V]) of the token after it."""
    n = kv[0][0].shape[0]
    hf, P = _infer_rows(cfg, params, [int(token)], [n], kv, trainable)
    return hf[0].astype(np.float64) @ P.lm_head("lm_head").astype(np.float64).T


def greedy_generate(cfg, params, prompt, n_new, trainable=None):
    """Greedy decoding: n_new tokens, each the arg max (lowest index on ties) of the previous step's logits.  Returns
    (tokens int32 [n_new], logits fp64 [n_new][V])."""
    kv = new_kv(cfg)
    logits = infer_prefill(cfg, params, prompt, kv, trainable)
    toks, lgs = [], []
    for _ in range(n_new):
        lgs.append(logits)
        toks.append(int(np.argmax(logits)))
        if len(toks) < n_new:
            logits = infer_decode(cfg, params, toks[-1], kv, trainable)
    return np.array(toks, np.int32), np.stack(lgs)


def zo_step(cfg, params, seed, eps, lr, ids=None, x=None, target=None, trainable=None, lr_smooth=None, lr_clip=None,
            stochastic=False):
    """One ZO-SGD step (Eq. 2 with q = 1, then Eq. 3), updating `params` in place.

    Entries of `params` that are PackedInt4 are frozen (their `trainable` flag must be False).
    Returns (L+, L-, g) as fp32."""
    eps = np.float32(eps)
    lp = forward(cfg, params, ids, x, target, seed, eps, trainable)
    lm = forward(cfg, params, ids, x, target, seed, -eps, trainable)
    g = projected_grad(lp, lm, eps)
    # one coefficient per learning-rate group (model, smoothing, clipping); the same g and u for all
    lrs = [lr, lr if lr_smooth is None else lr_smooth, lr if lr_clip is None else lr_clip]
    cs = [coeff(np.float32(v), g) for v in lrs]
    groups = param_groups(cfg)
    for i, w in enumerate(params):
        if isinstance(w, PackedInt4):
            continue
        if trainable is None or trainable[i]:
            update(w, seed, i, cs[groups[i]], stochastic)
    return lp, lm, g


def zo_step_multi(cfg, params, seeds, eps, lr, ids=None, x=None, target=None, trainable=None, lr_smooth=None, lr_clip=None,
                  stochastic=False):
    """One ZO-SGD step with q = len(seeds) directions (Eq. 2, then Eq. 3), updating `params` in place.

    Every direction's pair of losses is evaluated at the same, not yet updated, W; the estimate is the
    average (1/q) sum_i g_i u_i, so W <- W - sum_i (eta/q) g_i u_i.  Readings: the factor 1/q is folded
    into the step size once (eta_q = fl32(eta / q)); the q rank-one terms are applied in the order of
    `seeds`, one fp32 fused multiply-add each.  Returns [(L+, L-, g_i)] per direction."""
    q = len(seeds)
    eps = np.float32(eps)
    res = []
    for s in seeds:
        lp = forward(cfg, params, ids, x, target, s, eps, trainable)
        lm = forward(cfg, params, ids, x, target, s, -eps, trainable)
        res.append((lp, lm, projected_grad(lp, lm, eps)))
    lrs = [lr, lr if lr_smooth is None else lr_smooth, lr if lr_clip is None else lr_clip]
    lrq = [np.float32(np.float32(v) / np.float32(q)) for v in lrs]
    groups = param_groups(cfg)
    for i, w in enumerate(params):
        if isinstance(w, PackedInt4):
            continue
        if trainable is None or trainable[i]:
            update_multi(w, seeds, i, [coeff(lrq[groups[i]], g) for _, _, g in res], stochastic)
    return res


def lr_linear_decay(lr0, t, T):
    """Step size of iteration t = 0 .. T-1 under the linear-decay schedule of the hyperparameter table
    (pre-training); reading: eta_t = eta_0 (1 - t/T), reaching eta_0/T at the last iteration.  The
    fine-tuning runs use a constant step size."""
    return np.float32(float(np.float32(lr0)) * (1.0 - float(t) / float(T)))
