#!/usr/bin/env python3
"""Benchmark of the ZO-QAT step on one MI355X.

A "step" is one zo_step call: both quantized forwards of Eq. 2 at W +- eps u, the projected
gradient, and the seeded update of Eq. 3, on a batch of synthetic token ids with random-init
weights of the named shape, all resident in HBM before the timed region.

Prints ONE JSON line (rank 0): ZO steps/s, the roofline of the dominant kernel (the bf16 MFMA
GEMM of the fake-quantized linears, timed per launch with HIP events on the launch stream inside
the timed region), the update kernel's HBM rate, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # Llama-2-7B shape, W4A8 group 64, 8 x 1024 tokens (the configuration the metric is quoted on)
    "llama7b_w4a8_g64_8x1024": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                    w_bits=4, w_group=64, a_bits=8, B=8, S=1024),
    "llama7b_w2a16_g64_8x1024": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                     w_bits=2, w_group=64, a_bits=16, B=8, S=1024),
    "opt1p3b_w4a8_g128_16x512": dict(arch="opt", n_layers=24, d_model=2048, n_heads=32, d_ffn=8192, vocab=50272,
                                     w_bits=4, w_group=128, a_bits=8, B=16, S=512),
    # 13B shape, lightweight variant: everything frozen (linears as packed 4-bit codes + binary16 steps, group 128),
    # only the query / value projections trainable; per-token 4-bit activations; 4 x 2048 tokens
    "llama13b_lightweight_w4a4_g128_4x2048": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                  vocab=32000, w_bits=4, w_group=128, a_bits=4, B=4, S=2048, lightweight=1),
    # the paper's own quantizer settings (Eq. 5 / Eq. 4 as ZO-trained tensors, learning rates of the appendix table):
    # Llama-shaped weight-only keeps the clipping only; OPT-shaped W4A4 has smoothing and clipping
    "llama7b_w2a16_g64_clip_8x1024": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                          w_bits=2, w_group=64, a_bits=16, B=8, S=1024, learn_clip=1),
    "opt1p3b_w4a4_g128_smooth_clip_16x512": dict(arch="opt", n_layers=24, d_model=2048, n_heads=32, d_ffn=8192, vocab=50272,
                                                 w_bits=4, w_group=128, a_bits=4, B=16, S=512, learn_clip=1, learn_smooth=1),
    # the small-batch regime of the paper's fine-tuning runs (batch 1, a few hundred tokens): every linear takes the
    # fused kernel that builds the tiles of Q(W +- eps u) in registers; --no-fused times the quantize-once route
    "llama7b_w4a8_g64_1x128": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                   w_bits=4, w_group=64, a_bits=8, B=1, S=128),
    "llama7b_w4a8_g64_1x64": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                  w_bits=4, w_group=64, a_bits=8, B=1, S=64),
    "llama7b_w4a8_g64_1x32": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                  w_bits=4, w_group=64, a_bits=8, B=1, S=32),
    # between the two regimes (the fine-tuning table's 384-token sequences, batch 1 and 16): quantize once, then GEMMs
    "llama7b_w4a8_g64_1x256": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                   w_bits=4, w_group=64, a_bits=8, B=1, S=256),
    "llama7b_w4a8_g64_1x384": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                   w_bits=4, w_group=64, a_bits=8, B=1, S=384),
    "llama7b_w4a8_g64_16x384": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                    w_bits=4, w_group=64, a_bits=8, B=16, S=384),
    # the lightweight variant in the same regime: frozen linears expanded from their packed codes inside the kernel
    "llama13b_lightweight_w4a4_g128_1x128": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                 vocab=32000, w_bits=4, w_group=128, a_bits=4, B=1, S=128, lightweight=1),
    "llama13b_lightweight_w4a4_g128_1x64": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                vocab=32000, w_bits=4, w_group=128, a_bits=4, B=1, S=64, lightweight=1),
    "llama13b_lightweight_w4a4_g128_1x32": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                vocab=32000, w_bits=4, w_group=128, a_bits=4, B=1, S=32, lightweight=1),
    # the shapes of the paper's fine-tuning rows for the lightweight variant (efficiency section, GPU table: sequences of at
    # most 384 tokens, batch 1 and 16; its figures there are for another card and W2A16 g128: context only)
    "llama13b_lightweight_w4a4_g128_1x384": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                 vocab=32000, w_bits=4, w_group=128, a_bits=4, B=1, S=384, lightweight=1),
    "llama13b_lightweight_w4a4_g128_16x384": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                                                  vocab=32000, w_bits=4, w_group=128, a_bits=4, B=16, S=384, lightweight=1),
    # the trained model as a generator (efficiency section, on-device table: W4A4 inference, 384-token prompts): every quantized
    # linear stored as packed 4-bit codes, prompt pass over 384 tokens, then greedy decoding token by token
    "llama13b_w4a4_g128_generate_384": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824, vocab=32000,
                                            w_bits=4, w_group=128, a_bits=4, B=1, S=384, lightweight=1, generate=64),
    "llama7b_w4a4_g128_generate_384": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                           w_bits=4, w_group=128, a_bits=4, B=1, S=384, lightweight=1, generate=64),
    # per-channel weight steps (the weight setting of the W4A4 rows of the appendix's quantization settings) at the 7B shape:
    # with --mma int8 the quantized linears contract their integer codes and the loop has no rescale at all
    "llama7b_w4a8_perchannel_8x1024": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                           w_bits=4, w_group=0, a_bits=8, B=8, S=1024),
    "llama7b_w4a4_perchannel_8x1024": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
                                           w_bits=4, w_group=0, a_bits=4, B=8, S=1024),
    "tiny_w4a16_g64_8x128": dict(arch="llama", n_layers=4, d_model=512, n_heads=8, d_ffn=2048, vocab=4096,
                                 w_bits=4, w_group=64, a_bits=16, B=8, S=128),
}
# HBM-side bytes per launch of the GEMM kernel: counters cannot be read from inside the run, so the figure is the one
# the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this same command holds (profiles/zo_step_<workload>_hbm_traffic.txt,
# line "gemm_traffic_bytes_per_launch = ..."; it says how the counters were scaled by a plain copy of known size).  A workload
# without such a summary reports null; the summary is regenerated whenever the GEMM kernel or its launch order changes.
def measured_gemm_traffic(workload):
    path = os.path.join(ROOT, "profiles", "zo_step_%s_hbm_traffic.txt" % workload.replace("_g64_8x1024", ""))
    try:
        for line in open(path):
            if line.strip().startswith("gemm_traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


BREAKDOWN_STEPS = 2
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_INT8_TOPS = 5000.0        # MI355X dense int8 MFMA
PEAK_HBM_GBS = 8000.0
# plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (the fp32 vector peak of
# 157.3 TFLOP/s counts 2 flops per FMA and the packed two-per-lane forms, which this build does not use)
PEAK_ALU_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# lane-instructions of the fused small-M kernel per parameter: SQ_INSTS_VALU of a rocprofv3 counter pass over the 1 x 32 workload
# (profiles/zo_step_llama7b_w4a8_1x32_fused_kernel_valu.txt: 3.8297e7 wave-instructions x 64 lanes / 4.0475e7 parameters per launch)
FUSED_LANEOPS_PER_PARAM = 60.6


def gemm_flops_per_step(w):
    """2*M*N*K over every GEMM launch of one step (both branches): the algorithmic flops."""
    M, d, f, V, L = w["B"] * w["S"], w["d_model"], w["d_ffn"], w["vocab"], w["n_layers"]
    ffn = 3 * d * f if w["arch"] == "llama" else 2 * d * f
    per_fwd = L * (4 * d * d + ffn) + V * d
    return 2 * 2.0 * M * per_fwd


def attention_flops_per_step(w):
    B, S, d, L = w["B"], w["S"], w["d_model"], w["n_layers"]
    return 2 * L * B * 2 * 2.0 * d * S * (S + 1) / 2            # QK^T and PV over the causal half


def cpu_baseline(w):
    """The oracle, as it stands, timed on a bounded sample of the workload: one full ZO step of a
    1-layer model of the same widths and vocabulary on one sequence.  Extrapolated to the full
    depth and batch by the ratio of GEMM flops (the dominant term of the full workload)."""
    import numpy as np  # noqa: F401
    from oracle import zo_oracle as orc
    from paper_2509_00031_amd import synth
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = 1
    omp = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    arch = orc.ARCH_LLAMA if w["arch"] == "llama" else orc.ARCH_OPT
    cfg = orc.Config(arch, n_layers=1, d_model=w["d_model"], n_heads=w["n_heads"], d_ffn=w["d_ffn"], vocab=w["vocab"],
                     max_seq=w["S"], w_bits=w["w_bits"], w_group=w["w_group"], a_bits=w["a_bits"], act_dtype=1,
                     lightweight=w.get("lightweight", 0), learn_clip=w.get("learn_clip", 0), learn_smooth=w.get("learn_smooth", 0))
    shapes = orc.param_shapes(cfg)
    params = synth.model_params(shapes, 1234)
    if cfg.learn_clip or cfg.learn_smooth:
        orc.init_learned_params(cfg, params)
    trainable = None
    if w.get("lightweight"):
        trainable = [name.endswith(".wq") or name.endswith(".wv") for name, _, _ in shapes]
        params = [orc.pack_int4(p, w["w_group"]) if (q and not t) else p for p, t, (_, _, q) in zip(params, trainable, shapes)]
    ids = synth.token_ids(1, w["S"], w["vocab"], 5678)
    t0 = time.perf_counter()
    orc.zo_step(cfg, params, 0, 1e-3, 1e-6, ids=ids, trainable=trainable, lr_smooth=5e-6, lr_clip=1e-5)
    t_sample = time.perf_counter() - t0
    sample = dict(w, n_layers=1, B=1)
    ratio = gemm_flops_per_step(w) / gemm_flops_per_step(sample)
    est = t_sample * ratio
    return {"value": 1.0 / est, "unit": "steps/s", "cores": max(blas_threads, omp), "kind": "oracle",
            "sample": "one oracle zo_step of a 1-layer model of the same widths on 1 of %d sequences of %d tokens took "
                      "%.1f s; extrapolated by the GEMM-flop ratio full/sample = %.0f to %.0f s per full step"
                      % (w["B"], w["S"], t_sample, ratio, est)}


def bench_generate(args, w):
    """Prompt pass + greedy decoding on the packed model.  A "step" here is one generated token; value = decoded tokens / s."""
    import torch
    from paper_2509_00031_amd import binding as zo
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    S, n_new = w["S"], w["generate"]
    kv_len = S + n_new
    cfg = zo.make_config(zo.ARCH_LLAMA, n_layers=w["n_layers"], d_model=w["d_model"], n_heads=w["n_heads"], d_ffn=w["d_ffn"],
                         vocab=w["vocab"], max_seq=kv_len, w_bits=w["w_bits"], w_group=w["w_group"], a_bits=w["a_bits"],
                         act_dtype=zo.ACT_BF16, lightweight=1)
    n = zo.zo_num_params(cfg)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    kind = lambda i: (i - 1) % 9 if 1 <= i <= 9 * w["n_layers"] else -1
    params, code_bytes, other_bytes = [], 0, 0
    for i in range(n):
        numel = zo.zo_param_numel(cfg, i)
        t = torch.empty(numel, dtype=torch.float32, device=dev).normal_(0.0, 0.02, generator=gen)
        if numel == w["d_model"]:
            t.add_(1.0)
        if kind(i) in (1, 2, 3, 4, 6, 7, 8):            # every quantized linear: packed codes + binary16 step + int16 zero point per group
            K = w["d_ffn"] if kind(i) == 8 else w["d_model"]
            t = zo.zo_pack_weight_int4(t.view(numel // K, K), w["w_group"])
            code_bytes += numel // 2 + 4 * (numel // w["w_group"])
        elif i == n - 1:
            other_bytes += 4 * numel                     # the lm_head stays fp32 and is read once per token
        params.append(t)
    ctx = zo.Context(cfg, params, 1, S, trainable=[False] * n)
    prompt = torch.randint(0, w["vocab"], (S,), dtype=torch.int32, device=dev, generator=gen)
    kv = ctx.new_kv_cache(kv_len)
    tokens = torch.zeros(n_new, dtype=torch.int32, device=dev)
    logits = torch.empty(w["vocab"], dtype=torch.float32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for _ in range(max(args.warmup, 1)):
        ctx.zo_generate_greedy(prompt, n_new, kv, kv_len, tokens, logits)
    torch.cuda.synchronize()
    t_pre, t_gen = [], []
    for _ in range(args.steps):
        a, b, c_ = ev(), ev(), ev()
        a.record()
        ctx.zo_prefill(prompt, kv, kv_len, logits)
        b.record()
        ctx.zo_generate_greedy(prompt, n_new, kv, kv_len, tokens, logits)
        c_.record()
        torch.cuda.synchronize()
        t_pre.append(a.elapsed_time(b))
        t_gen.append(b.elapsed_time(c_))
    pre_ms = sorted(t_pre)[len(t_pre) // 2]
    gen_ms = sorted(t_gen)[len(t_gen) // 2]
    per_tok_ms = (gen_ms - pre_ms) / (n_new - 1)        # n_new - 1 cached steps follow the prompt pass
    bytes_per_tok = code_bytes + other_bytes
    ach = bytes_per_tok / (per_tok_ms * 1e-3) / 1e9
    res = {"metric": "decoded tokens/sec (greedy, batch 1, packed 4-bit model)", "value": 1e3 / per_tok_ms, "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": per_tok_ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "prompt_tokens": S, "generated_tokens": n_new, "w_bits": w["w_bits"], "w_group": w["w_group"],
                      "a_bits": w["a_bits"], "first_tokens": tokens[:4].cpu().tolist()},
           "prefill_ms": pre_ms, "prefill_tokens_per_s": S / (pre_ms * 1e-3),
           "roofline": {"bound": "hbm", "kernel": "decoding step (packed-codes small-M kernels + lm_head)", "achieved": ach, "peak": PEAK_HBM_GBS,
                        "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None, "bytes_per_token": bytes_per_tok,
                        "codes_bytes_per_token": code_bytes}}
    ctx.close()
    print(json.dumps(res))


def measured_ceilings(torch, zo):
    """What this card sustains with nothing in the way, measured in the same process (events on the launch stream): bf16
    matrix instructions on register-resident operands (zo_probe_mfma_only; the power-managed clock depends on the operand
    data, so both random and all-zero operands are timed), and an in-place read-modify-write stream over 1 GiB."""
    out = {}
    buf = None
    for name, zero in (("mfma_only_random_operands_tflops", 0), ("mfma_only_zero_operands_tflops", 1)):
        buf, _ = zo.zo_probe_mfma_only(512, 500, zero, buf)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        buf, flop = zo.zo_probe_mfma_only(512, 20000, zero, buf)
        e1.record()
        torch.cuda.synchronize()
        out[name] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    x = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    x.mul_(1.0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        x.mul_(1.0)
    e1.record()
    torch.cuda.synchronize()
    out["inplace_stream_gbs"] = 5 * 2.0 * x.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del x, buf
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_w4a8_g64_8x1024", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--directions", type=int, default=1,
                    help="q of Eq. 2: forward pairs per step (all at the same W), followed by one multi-direction update pass")
    ap.add_argument("--masters", choices=["f32", "f16", "f16sr"], default="f32",
                    help="storage of the master weights: fp32 (the benchmark configurations), IEEE binary16 rounded to nearest "
                         "even (f16) or stochastically (f16sr) in the update -- the 2 bytes per parameter of the paper's memory table")
    ap.add_argument("--no-fused", action="store_true", help="small token counts: quantize once and run the plain GEMM")
    ap.add_argument("--mma", choices=["bf16", "int8"], default="bf16",
                    help="contraction of the quantized linears: bf16 matrix instructions on de-quantized operands (the benchmark "
                         "configurations), or int8 matrix instructions on the integer codes (zo_config.mma)")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket launches with HIP events in the timed region")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the timed region copy 1 GiB device to device once (a plain copy of known size, "
                         "against which the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the ZO-QAT step on ONE GPU (seed-synchronous data parallelism across GPUs is a "
              "design note only); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_00031_amd import binding as zo

    w = WORKLOADS[args.workload]
    if w.get("generate"):
        return bench_generate(args, w)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    ceilings = None if args.no_profile else measured_ceilings(torch, zo)
    arch = zo.ARCH_LLAMA if w["arch"] == "llama" else zo.ARCH_OPT
    cfg = zo.make_config(arch, n_layers=w["n_layers"], d_model=w["d_model"], n_heads=w["n_heads"], d_ffn=w["d_ffn"],
                         vocab=w["vocab"], max_seq=w["S"], w_bits=w["w_bits"], w_group=w["w_group"], a_bits=w["a_bits"],
                         act_dtype=zo.ACT_BF16, lightweight=w.get("lightweight", 0), learn_clip=w.get("learn_clip", 0),
                         learn_smooth=w.get("learn_smooth", 0), no_fused=int(args.no_fused),
                         master_dtype=zo.MASTER_F16 if args.masters != "f32" else zo.MASTER_F32, master_round=int(args.masters == "f16sr"),
                         mma=zo.MMA_INT8 if args.mma == "int8" else zo.MMA_BF16)
    n = zo.zo_num_params(cfg)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    params = []
    n_params = 0
    trainable = None
    if w.get("lightweight"):
        # llama tensor order: tok_emb, then per layer 9 tensors (norm, wq, wk, wv, wo, norm, gate, up, down), final norm, head
        assert w["arch"] == "llama"
        kind = lambda i: (i - 1) % 9 if 1 <= i <= 9 * w["n_layers"] else -1
        trainable = [kind(i) in (1, 3) for i in range(n)]
        packed_kinds = (2, 4, 6, 7, 8)
    for i in range(n):
        numel = zo.zo_param_numel(cfg, i)
        t = torch.empty(numel, dtype=torch.float32 if args.masters == "f32" else torch.float16, device=dev)
        t.normal_(0.0, 0.02, generator=gen)
        if numel == w["d_model"]:                       # norm gains / small vectors: around one
            t.add_(1.0)
        if trainable is None or trainable[i]:
            n_params += numel
        elif kind(i) in packed_kinds:                   # frozen linear: keep only its packed 4-bit form
            K = w["d_ffn"] if kind(i) == 8 else w["d_model"]
            t = zo.zo_pack_weight_int4(t.float().view(numel // K, K), w["w_group"])
        params.append(t)
    B, S = w["B"], w["S"]
    ids = torch.randint(0, w["vocab"], (B, S), dtype=torch.int32, device=dev, generator=gen)
    ctx = zo.Context(cfg, params, B, S, trainable=trainable)
    eps, lr = 1e-3, 1e-6
    learned = bool(w.get("learn_clip") or w.get("learn_smooth"))
    if learned:
        ctx.zo_init_learned_params()              # the quantizer / smoothing tensors were filled with noise above
    lr_smooth, lr_clip = 5e-6, 1e-5               # appendix, hyperparameter table
    out6 = torch.zeros(6, dtype=torch.float32, device=dev)

    def one_step(seed):
        if args.directions > 1:
            q = args.directions
            return ctx.zo_step_multi(ids, None, B, S, [seed * q + i for i in range(q)], eps, lr, lr_smooth, lr_clip)[q - 1]
        if learned:
            return ctx.zo_step_groups(ids, None, B, S, seed, eps, lr, lr_smooth, lr_clip, out6)
        return ctx.zo_step(ids, None, B, S, seed=seed, eps=eps, lr=lr)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    # Timed region: only the launches of the kernel the roofline object is about (the GEMM; the fused kernels on the
    # small-batch workloads) are bracketed with events -- a bracket leaves the stream idle for a few microseconds, and a
    # step has about a thousand launches.  The per-category breakdown and the update kernel's figure come from
    # BREAKDOWN_STEPS further steps, after the timed region, with every launch bracketed.
    ROOFLINE_CATEGORIES = ("gemm", "fused_linear", "fused_int4_linear")
    if not args.no_profile:
        ctx.zo_profile_begin_mask(ROOFLINE_CATEGORIES)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # one event per step boundary, same stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        out = one_step(args.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = None if args.no_profile else ctx.zo_profile_end()
    losses = out.cpu().tolist()
    prof_all = None
    if not args.no_profile:
        ctx.zo_profile_begin()
        for i in range(BREAKDOWN_STEPS):
            one_step(args.warmup + args.steps + i)
        prof_all = ctx.zo_profile_end()

    ms_per_step = 1e3 * elapsed / args.steps
    res = {
        "metric": "ZO steps/sec (2 quantized fwd + update)", "value": args.steps / elapsed, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8" if args.mma == "int8" else "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "mma": args.mma, "tokens_per_step": B * S, "trainable_params": n_params,
                   "w_bits": w["w_bits"], "w_group": w["w_group"], "a_bits": w["a_bits"], "eps": eps, "lr": lr,
                   "directions": args.directions, "masters": args.masters,
                   "last_step": {"loss_plus": losses[0], "loss_minus": losses[1], "g": losses[2]}},
    }
    gflops = gemm_flops_per_step(w) * args.directions
    if prof:
        gemm_ms, gemm_launches = prof["gemm"]
        avg_ms = gemm_ms / max(gemm_launches, 1)
        flops_per_launch = gflops * args.steps / max(gemm_launches, 1)
        achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
        res["roofline"] = {"bound": "mfma", "kernel": "zo_gemm_bf16_dma_kernel<bf16, 8 waves, BK 64, 2 stages>", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                           "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_gemm_traffic(args.workload),
                           "launches": gemm_launches, "avg_launch_ms": avg_ms,
                           "flops_per_launch": flops_per_launch}
        res["gemm_tflops"] = achieved
        if args.mma == "int8":
            # the quantized linears run zo_gemm_i8_kernel (98.8 % of the operations at the 7B shape; the un-quantized lm_head
            # keeps its bf16 launch, counted with them): priced against the dense int8 peak
            res["roofline"].update({"kernel": "zo_gemm_i8_kernel<8 waves, 128-byte K tiles, 2 stages> (+ the bf16 lm_head launch)",
                                    "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": achieved / PEAK_INT8_TOPS, "traffic": None})
        fused_ms, fused_launches = prof["fused_linear"]
        int4_ms, int4_launches = prof["fused_int4_linear"]
        if int4_launches > 0 and int4_ms >= fused_ms:
            # lightweight variant at a small token count: the kernel that expands the packed codes dominates; it moves
            # 0.5 B of codes per weight (+ 4 B per group of step and zero point) and nothing else of that order
            d, f, L, g = w["d_model"], w["d_ffn"], w["n_layers"], w["w_group"]
            packed_weights = L * (2 * d * d + 3 * d * f)              # wk, wo, gate, up, down
            avg_ms = int4_ms / int4_launches
            bytes_per_launch = (0.5 + 4.0 / g) * packed_weights * args.steps / int4_launches
            ach = bytes_per_launch / (avg_ms * 1e-3) / 1e9
            res["roofline"] = {"bound": "hbm", "kernel": "zo_int4_gemm_fused_kernel", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": ach / PEAK_HBM_GBS, "traffic": None, "launches": int4_launches, "avg_launch_ms": avg_ms,
                               "bytes_per_launch": bytes_per_launch}
            res["gemm_tflops"] = gflops * args.steps / ((fused_ms + int4_ms) * 1e-3) / 1e12
        elif fused_launches > 0:
            # small-M route: every linear went through the fused kernel, which is bound by the plain-ALU tile build
            d, f, V, L = w["d_model"], w["d_ffn"], w["vocab"], w["n_layers"]
            lin_params = L * (4 * d * d + (3 if w["arch"] == "llama" else 2) * d * f) + V * d
            avg_ms = fused_ms / fused_launches
            params_per_launch = lin_params * args.steps / fused_launches
            ach = FUSED_LANEOPS_PER_PARAM * params_per_launch / (avg_ms * 1e-3) / 1e12
            res["roofline"] = {"bound": "alu", "kernel": "zo_fq_gemm_fused_kernel", "achieved": ach, "peak": PEAK_ALU_TLANEOPS,
                               "unit": "Tlane-op/s", "frac": ach / PEAK_ALU_TLANEOPS, "traffic": None,
                               "launches": fused_launches, "avg_launch_ms": avg_ms, "params_per_launch": params_per_launch,
                               "master_GBps": 4.0 * params_per_launch / (avg_ms * 1e-3) / 1e9}
            res["gemm_tflops"] = gflops * args.steps / (fused_ms * 1e-3) / 1e12
        upd_ms, upd_groups = prof_all["update"]
        upd_bpp = 8 if args.masters == "f32" else 4          # one read + one write of every trainable master
        upd_gbs = upd_bpp * n_params * upd_groups / (upd_ms * 1e-3) / 1e9 if upd_ms > 0 else None
        res["update_kernel"] = {"bound": "hbm", "achieved": upd_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": upd_gbs / PEAK_HBM_GBS if upd_gbs else None, "bytes_per_param": upd_bpp,
                                "ms_per_step": upd_ms / max(upd_groups, 1)}
        res["breakdown_ms_per_step"] = {k: v[0] / BREAKDOWN_STEPS for k, v in prof_all.items()}
        if ceilings:
            # next to the published peaks: the same figures against what the card sustains in this process with nothing in the way
            res["measured_ceilings"] = ceilings
            if res["roofline"]["bound"] == "mfma" and args.mma == "bf16":
                res["roofline"]["frac_of_measured_mfma_only"] = res["roofline"]["achieved"] / ceilings["mfma_only_random_operands_tflops"]
            if upd_gbs:
                res["update_kernel"]["frac_of_measured_stream"] = upd_gbs / ceilings["inplace_stream_gbs"]
        if res["roofline"]["bound"] == "mfma":
            # The weights are quantized once per step into the operand buffers (the prologue of every fake-quantized GEMM):
            # "frac" is the GEMM kernel alone, "frac_with_prologue" counts 2 M N K against GEMM time + weight-quantizer time
            # (timed region's GEMM time per step + the weight-quantizer time of the fully bracketed steps).
            gemm_ms_step = gemm_ms / args.steps
            wq_ms_step = res["breakdown_ms_per_step"]["weight_quant"]
            with_pro = gflops / ((gemm_ms_step + wq_ms_step) * 1e-3) / 1e12
            res["roofline"].update({"frac_gemm_only": res["roofline"]["frac"], "frac_with_prologue": with_pro / res["roofline"]["peak"],
                                    "achieved_with_prologue": with_pro, "prologue": "zo_fq_weight_kernel (quantize once per step)",
                                    "prologue_ms_per_step": wq_ms_step, "gemm_ms_per_step": gemm_ms_step,
                                    "note": "frac = GEMM kernel alone (2MNK / its launch time); frac_with_prologue = 2MNK / (GEMM + weight "
                                            "quantizer time); the 0.50 target is compared with both"})
        res["breakdown_source"] = "%d further steps after the timed region, every launch bracketed by events" % BREAKDOWN_STEPS
    res["step_flops"] = gflops + attention_flops_per_step(w) * args.directions
    res["step_tflops"] = res["step_flops"] / (ms_per_step * 1e-3) / 1e12
    ctx.close()
    del params, ctx
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
