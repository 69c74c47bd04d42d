"""Pins for the oracle's model-level forward (CPU only).  The paper does not define the
transformer around the quantized linears; with quantization off and no perturbation the
oracle must equal the same decoder assembled from torch.nn.functional routines in fp64."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _t(a):
    return torch.from_numpy(np.asarray(a)).double()


def _torch_decoder(cfg, params, ids):
    names = [n for n, _, _ in orc.param_shapes(cfg)]
    P = {n: _t(p) for n, p in zip(names, params)}
    B, S = ids.shape
    d, H = cfg.d_model, cfg.n_heads
    dh = d // H
    tid = torch.from_numpy(ids).long()
    x = F.embedding(tid, P["tok_emb"])
    if cfg.arch == orc.ARCH_OPT:
        x = x + P["pos_emb"][:S][None]
    else:
        inv = 10000.0 ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
        rot = torch.polar(torch.ones(S, dh // 2, dtype=torch.float64),
                          torch.arange(S, dtype=torch.float64)[:, None] * inv[None])      # e^{i pos w}

        def rope(t):                                  # t [B,S,H,dh]; pair (i, i+dh/2) as a complex number
            c = torch.complex(t[..., : dh // 2], t[..., dh // 2:]) * rot[None, :, None, :]
            return torch.cat([c.real, c.imag], -1)
    for l in range(cfg.n_layers):
        p = "l%d." % l
        if cfg.arch == orc.ARCH_LLAMA:
            h = F.rms_norm(x, (d,), P[p + "attn_norm"], 1e-5)
            q, k, v = (F.linear(h, P[p + n]).view(B, S, H, dh) for n in ("wq", "wk", "wv"))
            q, k = rope(q), rope(k)
        else:
            h = F.layer_norm(x, (d,), P[p + "ln1_g"], P[p + "ln1_b"], 1e-5)
            q, k, v = (F.linear(h, P[p + "w" + n], P[p + "b" + n]).view(B, S, H, dh) for n in "qkv")
        a = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2), is_causal=True)
        a = a.transpose(1, 2).reshape(B, S, d)
        if cfg.arch == orc.ARCH_LLAMA:
            x = x + F.linear(a, P[p + "wo"])
            h = F.rms_norm(x, (d,), P[p + "ffn_norm"], 1e-5)
            x = x + F.linear(F.silu(F.linear(h, P[p + "w_gate"])) * F.linear(h, P[p + "w_up"]), P[p + "w_down"])
        else:
            x = x + F.linear(a, P[p + "wo"], P[p + "bo"])
            h = F.layer_norm(x, (d,), P[p + "ln2_g"], P[p + "ln2_b"], 1e-5)
            x = x + F.linear(F.relu(F.linear(h, P[p + "fc1"], P[p + "b1"])), P[p + "fc2"], P[p + "b2"])
    if cfg.arch == orc.ARCH_LLAMA:
        x = F.rms_norm(x, (d,), P["final_norm"], 1e-5)
    else:
        x = F.layer_norm(x, (d,), P["final_ln_g"], P["final_ln_b"], 1e-5)
    logits = F.linear(x, P["lm_head"])
    loss = F.cross_entropy(logits[:, :-1].reshape(-1, cfg.vocab), tid[:, 1:].reshape(-1))
    return logits.reshape(B * S, -1).numpy(), float(loss)


def _tiny(arch, **kw):
    base = dict(n_layers=2, d_model=64, n_heads=4, d_ffn=128, vocab=97, max_seq=16,
                w_bits=0, w_group=0, a_bits=16, act_dtype=0)
    base.update(kw)
    return orc.Config(arch, **base)


def test_llama_shaped_forward_matches_torch_functional():
    cfg = _tiny(orc.ARCH_LLAMA)
    params = synth.model_params(orc.param_shapes(cfg), 1)
    params = [p * (5.0 if p.ndim == 2 else 1.0) for p in params]        # make attention non-trivial
    ids = synth.token_ids(2, 12, cfg.vocab, 2)
    trace = {}
    loss = orc.forward(cfg, params, ids=ids, trace=trace)
    logits, ref = _torch_decoder(cfg, params, ids)
    assert np.abs(trace["logits"] - logits).max() < 2e-5               # fp32 storage between ops
    assert abs(float(loss) - ref) < 1e-5


def test_opt_shaped_forward_matches_torch_functional():
    cfg = _tiny(orc.ARCH_OPT)
    params = synth.model_params(orc.param_shapes(cfg), 3)
    params = [p * (5.0 if p.ndim == 2 else 1.0) for p in params]
    ids = synth.token_ids(3, 9, cfg.vocab, 4)
    trace = {}
    loss = orc.forward(cfg, params, ids=ids, trace=trace)
    logits, ref = _torch_decoder(cfg, params, ids)
    assert np.abs(trace["logits"] - logits).max() < 2e-5
    assert abs(float(loss) - ref) < 1e-5


def test_loss_at_random_init_is_log_vocab():
    cfg = _tiny(orc.ARCH_LLAMA, w_bits=4, w_group=32, a_bits=8)
    params = synth.model_params(orc.param_shapes(cfg), 5)
    ids = synth.token_ids(2, 16, cfg.vocab, 6)
    loss = orc.forward(cfg, params, ids=ids, seed=1, eps_signed=1e-3)
    assert abs(float(loss) - np.log(cfg.vocab)) < 0.1


def test_quantized_linear_config_is_quantizers_plus_triple_loop():
    cfg = orc.Config(orc.ARCH_LINEAR, d_model=64, d_ffn=48, w_bits=4, w_group=32, a_bits=8)
    W = synth.weights((48, 64), 7)
    x = synth.activations((5, 64), 8)
    tgt = synth.activations((5, 48), 9)
    eps = np.float32(1e-3)
    trace = {}
    loss = orc.forward(cfg, [W], x=x, target=tgt, seed=3, eps_signed=eps, trace=trace)
    what = orc.fakequant_weight(W, 4, 32, seed=3, tensor_id=0, eps_signed=eps)["what"]
    xhat = orc.fakequant_act(x, 8)["xhat"]
    y = orc.linear(xhat, what)
    assert np.array_equal(trace["y"], y.astype(np.float32))
    assert loss == np.float32(np.mean((y.astype(np.float32).astype(np.float64) - tgt) ** 2))


def test_bf16_mode_rounds_every_stored_activation():
    cfg = _tiny(orc.ARCH_LLAMA, w_bits=4, w_group=32, a_bits=8, act_dtype=1)
    params = synth.model_params(orc.param_shapes(cfg), 10)
    ids = synth.token_ids(2, 8, cfg.vocab, 11)
    trace = {}
    orc.forward(cfg, params, ids=ids, seed=2, eps_signed=1e-3, trace=trace)
    for name, val in trace.items():
        if name != "logits":
            assert np.array_equal(val, orc.bf16_round(val)), name


def test_zo_step_moves_every_trainable_tensor_along_minus_c_z():
    cfg = _tiny(orc.ARCH_OPT, n_layers=1, w_bits=4, w_group=32, a_bits=8)
    shapes = orc.param_shapes(cfg)
    params = synth.model_params(shapes, 12)
    before = [p.copy() for p in params]
    ids = synth.token_ids(2, 8, cfg.vocab, 13)
    trainable = [name.endswith("wq") or name.endswith("wv") for name, _, _ in shapes]
    lp, lm, g = orc.zo_step(cfg, params, seed=5, eps=1e-3, lr=1e-2, ids=ids, trainable=trainable)
    assert g == orc.projected_grad(lp, lm, np.float32(1e-3)) and g != 0
    c = orc.coeff(np.float32(1e-2), g)
    for i, (p0, p1) in enumerate(zip(before, params)):
        if trainable[i]:
            want = orc.update(p0.copy(), 5, i, c)
            assert np.array_equal(p1, want) and not np.array_equal(p1, p0)
        else:
            assert np.array_equal(p1, p0)
    # frozen tensors are not perturbed in the forwards either
    l_all = orc.forward(cfg, before, ids=ids, seed=5, eps_signed=1e-3)
    assert l_all != lp
