#!/usr/bin/env python3
"""Benchmark of the speculative-decoding verify step on one MI355X.

One "step" is one whole verify step: 28 decoder layers over the B*(gamma+1)
new positions (massv_verify_layers), the vocabulary projection (massv_lm_head_logits) and accept /
resample (massv_spec_accept) -- every call goes through the C ABI of libmassv_verify.so.  Inputs are synthetic and
resident in HBM before the timed region.

    python bench.py [--steps K] [--warmup W] [--workload NAME] [--no-extra] [--no-cpu]

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gateup_kernel_hbm_traffic.json")
KERNEL_SOURCES = ["paper_2505_10526_amd/csrc/gemm.hip", "paper_2505_10526_amd/csrc/common.h",
                  "paper_2505_10526_amd/csrc/kernels.h"]


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch of the gate/up kernel from the stored FETCH_SIZE / WRITE_SIZE counter runs
    (profiles/), or None when they were taken for another workload or the kernel's sources have changed."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
        if t.get("workload") != workload or t.get("kernel_source_sha256") != kernel_source_hash():
            return None
        return int(t["fetch_kib_per_dispatch"] * 1024 * t["fetch_scale"] + t["write_kib_per_dispatch"] * 1024 * t["write_scale"])
    except Exception:
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen7b_full",
                    choices=["qwen7b_full", "qwen7b_layer", "gemma12b_layer", "sd_iteration"])
    ap.add_argument("--layers", type=int, default=None, help="override the layer count (debugging)")
    ap.add_argument("--temperature", type=float, default=None, help="override the workload's sampling temperature")
    ap.add_argument("--no-extra", action="store_true", help="skip the attention/accept bandwidth section")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU checker timing")
    ap.add_argument("--only", default=None, choices=["linear_prefill", "prefill_attention"],
                    help="run just this compute-bound extra and print its record (for profiler runs of that kernel)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device copies (a kernel of known traffic, for scaling profiler byte counters)")
    return ap.parse_args()


WORKLOADS = {
    # full 28-layer Qwen2.5-VL-7B-shaped verify step (the headline workload)
    "qwen7b_full": dict(shape="QWEN7B", layers=28, batch=8, gamma=5, kv_lo=1024, kv_hi=2048,
                        img_lo=256, img_hi=1024, noise=1.5, temperature=0.0,
                        label="Qwen2.5-VL-7B-shaped full verify step: 28 layers + lm_head + accept, "
                              "B=8, gamma=5, kv_len U[1024,2048], 256-1024 image rows, T=0"),
    # one layer + lm_head + accept at batch 1
    "qwen7b_layer": dict(shape="QWEN7B", layers=1, batch=1, gamma=5, kv_lo=1024, kv_hi=1024,
                         img_lo=700, img_hi=700, noise=1.5, temperature=0.0,
                         label="one Qwen2.5-VL-7B-shaped layer + lm_head + accept, B=1, gamma=5, KV 1024, T=0"),
    # Gemma3-12B-shaped layer
    "gemma12b_layer": dict(shape="GEMMA12B", layers=1, batch=4, gamma=5, kv_lo=4096, kv_hi=4096,
                           img_lo=256, img_hi=256, noise=2.0, temperature=0.0,
                           label="one Gemma3-12B-shaped layer + lm_head + accept, B=4, gamma=5, KV 4096, T=0"),
}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_10526_amd import binding, synth
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_10526_amd import build
        build.build(verbose=False)
    binding.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.only:
        g0 = torch.Generator(device=dev)
        g0.manual_seed(args.seed + 1)
        fn = linear_prefill if args.only == "linear_prefill" else prefill_attention_bench
        print(json.dumps({args.only: fn(torch, binding, synth, dev, g0)}))
        return
    if args.workload == "sd_iteration":
        print(json.dumps(iteration_bench(torch, binding, synth, dev, args)))
        return
    lin = pfa = None
    if not args.no_extra:
        g0 = torch.Generator(device=dev)
        g0.manual_seed(args.seed + 1)
        lin = linear_prefill(torch, binding, synth, dev, g0)
        pfa = prefill_attention_bench(torch, binding, synth, dev, g0)
    wl = dict(WORKLOADS[args.workload])
    if args.layers:
        wl["layers"] = args.layers
    if args.temperature is not None:
        wl["temperature"] = float(args.temperature)
    shape = getattr(synth, wl["shape"])
    B, gamma, N = wl["batch"], wl["gamma"], wl["layers"]
    Q, M = gamma + 1, wl["batch"] * (gamma + 1)
    H, F, V, d = shape.hidden, shape.mlp, shape.vocab, shape.head_dim
    nq, nkv = shape.n_q_heads * d, shape.n_kv_heads * d

    # ---------------- synthetic inputs, generated on the device ----------------
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    bf = torch.bfloat16

    def randn(*s, std=1.0, mean=0.0):
        return (torch.randn(*s, generator=gen, device=dev, dtype=torch.float32) * std + mean).to(bf)

    rng = np.random.default_rng(args.seed)
    kv_len_h = rng.integers(wl["kv_lo"], wl["kv_hi"] + 1, B).astype(np.int32)
    n_img_h = rng.integers(wl["img_lo"], wl["img_hi"] + 1, B).astype(np.int32)
    l_max = (int(wl["kv_hi"]) + Q + 31) // 32 * 32
    kv_len = torch.from_numpy(kv_len_h).to(dev)
    pos = torch.from_numpy(synth.positions(kv_len_h, n_img_h, Q)).to(dev)

    layers = []
    raw0 = None                                  # layer 0 before packing, kept for the parity leg
    for li in range(N):
        w = {"ln1": randn(H, std=0.1, mean=1.0), "wq": randn(nq, H, std=0.02), "wk": randn(nkv, H, std=0.02),
             "wv": randn(nkv, H, std=0.02), "wo": randn(H, nq, std=0.02), "ln2": randn(H, std=0.1, mean=1.0),
             "wg": randn(F, H, std=0.02), "wu": randn(F, H, std=0.02), "wd": randn(H, F, std=0.02),
             "bq": None, "bk": None, "bv": None}
        if shape.qkv_bias:
            w.update(bq=randn(nq, std=0.02), bk=randn(nkv, std=0.02), bv=randn(nkv, std=0.02))
        kc = randn(B, shape.n_kv_heads, l_max, d)
        vc_rows = randn(B, shape.n_kv_heads, l_max, d)
        for b in range(B):                       # image rows carry a wider spread (input recipe)
            kc[b, :, : int(n_img_h[b])] *= 1.5
        if li == 0 and not args.no_cpu:
            raw0 = {"w": w, "k": kc.clone(), "v": vc_rows}
        vc = binding.v_cache_pack(vc_rows)
        kc = binding.k_cache_pack(kc)
        w = binding.pack_layer_weights(w)           # projection matrices -> streaming layout (load-time step)
        layers.append((w, binding.layer_weights(w), kc, vc))
    final_norm = randn(H, std=0.1, mean=1.0)
    w_lm_rows = randn(V, H, std=0.02)
    w_lm = binding.weight_pack(w_lm_rows)
    if args.no_cpu:
        del w_lm_rows
    x0 = randn(B, Q, H)
    x = torch.empty_like(x0)
    logits = torch.empty((M, V), dtype=torch.float32, device=dev)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    out_tok = torch.empty((B, Q), dtype=torch.int32, device=dev)

    cfg = binding.LayerConfig(H, shape.n_q_heads, shape.n_kv_heads, d, F, shape.act, shape.qkv_bias,
                              shape.norm_eps, shape.rope_theta)
    desc = binding.layer_desc(cfg, B, Q, l_max, binding.BF16)
    ws_bytes = max(binding.verify_layer_workspace(desc),
                   binding.load().massv_lm_head_logits_workspace(M, H, V, binding.BF16),
                   binding.load().massv_lm_head_greedy_accept_workspace(B, gamma, H, V, binding.BF16),
                   binding.load().massv_spec_accept_workspace(B, gamma, V))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    T = wl["temperature"]

    stack = binding.LayerStack([lw for (_, lw, _, _) in layers], [kc for (_, _, kc, _) in layers],
                               [vc for (_, _, _, vc) in layers])

    def forward():
        x.copy_(x0)
        binding.verify_layers(cfg, stack, x, pos, kv_len, l_max, ws=ws, desc=desc)      # all N layers, one call
        binding.lm_head_logits(x.view(M, H), final_norm, w_lm, shape.norm_eps, out=logits, ws=ws)

    # draft logits / tokens: the drafter's output is an INPUT of the verify step.  It is derived once from the
    # target logits (target + N(0, noise)), outside the timed region.
    forward()
    torch.cuda.synchronize()
    tl = logits.view(B, Q, V)
    draft_logits = (tl[:, :gamma] + torch.randn(B, gamma, V, generator=gen, device=dev) * wl["noise"]).contiguous()
    draft_tokens = draft_logits.argmax(-1).to(torch.int32).contiguous()
    uniforms = torch.rand(B, Q, generator=gen, device=dev).clamp_(max=1 - 2 ** -24)

    def step():
        forward()
        binding.spec_accept(tl, draft_logits if T > 0 else None, draft_tokens, uniforms if T > 0 else None, T,
                            n_accepted=n_acc, out_tokens=out_tok, ws=ws)

    # ---------------- timed region ----------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # one gate/up launch per step (the first layer's) carries the caller's events -> live kernel duration
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:
        a.record(); b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        x.copy_(x0)
        binding.trace_kernel(binding.K_GATEUP, ev[s][0], ev[s][1])
        binding.verify_layers(cfg, stack, x, pos, kv_len, l_max, ws=ws, desc=desc)
        binding.lm_head_logits(x.view(M, H), final_norm, w_lm, shape.norm_eps, out=logits, ws=ws)
        binding.spec_accept(tl, draft_logits if T > 0 else None, draft_tokens, uniforms if T > 0 else None, T,
                            n_accepted=n_acc, out_tokens=out_tok, ws=ws)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    emitted = int((n_acc + 1).sum().item())
    tokens_per_s = emitted / (ms_per_step * 1e-3)
    k_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))

    # the same step with the vocabulary projection and the T = 0 accept rule fused (no logits written)
    fused_ms = None
    if T == 0:
        n_f, out_f = torch.empty_like(n_acc), torch.empty_like(out_tok)
        def fused_step():
            x.copy_(x0)
            binding.verify_layers(cfg, stack, x, pos, kv_len, l_max, ws=ws, desc=desc)
            binding.lm_head_greedy_accept(x, final_norm, w_lm, draft_tokens, shape.norm_eps, n_accepted=n_f, out_tokens=out_f, ws=ws)
        for _ in range(args.warmup):
            fused_step()
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for _ in range(args.steps):
            fused_step()
        torch.cuda.synchronize()
        fused_ms = (time.perf_counter() - tf0) * 1e3 / args.steps
        if not (torch.equal(n_f, n_acc) and torch.equal(out_f, out_tok)):
            print("bench.py: fused greedy step disagrees with the separate calls", file=sys.stderr)
            sys.exit(1)

    # ---------------- roofline of the dominant kernel: gate/up projection ----------------
    gateup_bytes = 2 * F * H * 2 + M * H * 2 + M * F * 2          # Wg, Wu (bf16) + X read + H written
    weight_bytes_step = N * (nq * H + 2 * nkv * H + H * nq + 3 * F * H) * 2 + V * H * 2
    achieved = gateup_bytes / (k_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "gemm_stream_kernel<MT,NT,EPI_GATED> (gate/up projection + activation)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(args.workload),
                "bytes_per_launch": gateup_bytes, "avg_launch_us": round(k_ms * 1e3, 2),
                "launches_timed": len(ev),
                "achieved_TFLOPs": round(2.0 * M * 2 * F * H / (k_ms * 1e-3) / 1e12, 1),
                "mfma_cap_TFLOPs_at_this_M": round(M * HBM_PEAK_GBS / 1e3, 1),     # M flops per weight byte x 8 TB/s
                "step_weight_stream_GBps": round(weight_bytes_step / (ms_per_step * 1e-3) / 1e9, 1)}
    # the whole step against the same roof: every byte the step has to move once (weights, the caches of all layers,
    # the fp32 logits written and read back by the accept call)
    kv_bytes_step = N * int(sum(2 * (int(L) + Q) * nkv * 2 for L in kv_len_h))
    logit_bytes_step = 2 * M * V * 4
    step_bytes = weight_bytes_step + kv_bytes_step + logit_bytes_step
    roofline["whole_step"] = {"what": "all launches of one step; the figure above is the gate/up kernel's alone",
                              "bytes": step_bytes, "achieved": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                              "unit": "GB/s", "frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # "peaked" variant of the same step: target logits x 8 before the same draft noise is added, which puts the
    # accepted lengths in the regime the paper reports (tau 2.5-3.3) instead of ~0; the step time does not depend
    # on the logit values, so only the accept call is repeated
    tl8 = (tl * 8.0).contiguous()
    dl8 = (tl8[:, :gamma] + (draft_logits - tl[:, :gamma])).contiguous()
    dt8 = dl8.argmax(-1).to(torch.int32).contiguous()
    n8 = torch.empty_like(n_acc)
    binding.spec_accept(tl8, dl8 if T > 0 else None, dt8, uniforms if T > 0 else None, T, n_accepted=n8,
                        out_tokens=torch.empty_like(out_tok), ws=ws)
    emitted8 = int((n8 + 1).sum().item())
    del tl8, dl8

    result = {
        "metric": "verified tokens/sec per verify step (7B-shape, gamma=5); attention+accept HBM GB/s",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl["label"], "layers": N, "batch": B, "gamma": gamma, "rows": M,
                   "kv_len": [int(v) for v in kv_len_h], "l_max": l_max, "temperature": T,
                   "draft_noise_std": wl["noise"], "launch": "eager, one stream"},
        "positions_per_s": round(M / (ms_per_step * 1e-3), 1),
        "mean_emitted_per_sequence": round(emitted / B, 3),
        "fused_greedy_ms_per_step": None if fused_ms is None else round(fused_ms, 4),
        "peaked_variant": {"what": "target logits x 8, same draft noise (synthetic)", "mean_emitted_per_sequence": round(emitted8 / B, 3),
                           "tokens_per_s": round(emitted8 / (ms_per_step * 1e-3), 1)},
        "roofline": roofline,
    }

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_extra:
        result["extra"] = extra_bandwidth(torch, binding, synth, dev, gen)
        result["extra"]["linear_prefill"] = lin
        result["extra"]["prefill_attention"] = pfa
    if not args.no_cpu:
        par, cpu = cpu_legs(torch, binding, wl, shape, cfg, raw0, layers[0], x0, x, pos, kv_len, kv_len_h, l_max,
                            final_norm, w_lm_rows, logits, draft_logits, draft_tokens, uniforms, n_acc, out_tok, T, ws)
        result["parity"] = par
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


class DeviceModel:
    """A random-weight decoder stack with embedding table, vocabulary projection and a KV cache, on the device."""

    def __init__(self, torch, binding, shape, n_layers, B, l_max, gen, dev):
        bf = torch.bfloat16
        H, F, d = shape.hidden, shape.mlp, shape.head_dim
        nq, nkv = shape.n_q_heads * d, shape.n_kv_heads * d

        def randn(*s, std=1.0, mean=0.0):
            return (torch.randn(*s, generator=gen, device=dev, dtype=torch.float32) * std + mean).to(bf)

        ws, ks, vs = [], [], []
        for _ in range(n_layers):
            w = {"ln1": randn(H, std=0.1, mean=1.0), "wq": randn(nq, H, std=0.02), "wk": randn(nkv, H, std=0.02),
                 "wv": randn(nkv, H, std=0.02), "wo": randn(H, nq, std=0.02), "ln2": randn(H, std=0.1, mean=1.0),
                 "wg": randn(F, H, std=0.02), "wu": randn(F, H, std=0.02), "wd": randn(H, F, std=0.02),
                 "bq": None, "bk": None, "bv": None}
            if shape.qkv_bias:
                w.update(bq=randn(nq, std=0.02), bk=randn(nkv, std=0.02), bv=randn(nkv, std=0.02))
            ws.append(binding.pack_layer_weights(w))
            ks.append(binding.k_cache_pack(randn(B, shape.n_kv_heads, l_max, d)))
            vs.append(binding.v_cache_pack(randn(B, shape.n_kv_heads, l_max, d)))
        self.shape, self.l_max = shape, l_max
        self.stack = binding.LayerStack(ws, ks, vs)
        self.final_norm = randn(H, std=0.1, mean=1.0)
        self.w_lm = binding.weight_pack(randn(shape.vocab, H, std=0.02))
        self.table = randn(shape.vocab, H)
        self.cfg = binding.LayerConfig(H, shape.n_q_heads, shape.n_kv_heads, d, F, shape.act, shape.qkv_bias,
                                       shape.norm_eps, shape.rope_theta)
        self.weight_bytes = n_layers * (nq * H + 2 * nkv * H + H * nq + 3 * F * H) * 2 + shape.vocab * H * 2


def iteration_bench(torch, binding, synth, dev, args):
    """One whole speculative-decoding iteration (paper Section 2.1) at the 7B-target / 1.5B-drafter shapes:
    gamma drafter decode steps (embedding, 28 layers at one query position, vocabulary projection, draw),
    then the target's verify pass over gamma+1 positions and the accept rule.  Random weights: acceptance
    is near zero, so tokens/s here is a floor; the per-part times and their ratio are the result."""
    B, gamma, T = 8, 5, float(args.temperature or 0.0)
    Q = gamma + 1
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    rng = np.random.default_rng(args.seed)
    kv_len_h = rng.integers(1024, 2049, B).astype(np.int32)
    n_img_h = rng.integers(256, 1025, B).astype(np.int32)
    l_max = (2048 + Q + 31) // 32 * 32
    n_layers = args.layers or 28
    tgt = DeviceModel(torch, binding, synth.QWEN7B, n_layers, B, l_max, gen, dev)
    drf = DeviceModel(torch, binding, synth.QWEN1P5B, n_layers, B, l_max, gen, dev)
    V = tgt.shape.vocab
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    kv_t, pos_t = i32(kv_len_h), i32(synth.positions(kv_len_h, n_img_h, Q))
    kv_d = [i32(kv_len_h + i) for i in range(gamma)]
    pos_d = [i32(synth.positions(kv_len_h + i, n_img_h, 1)) for i in range(gamma)]
    last = torch.randint(0, V, (B,), generator=gen, device=dev, dtype=torch.int32)
    uni_d = torch.rand(gamma, B, 1, generator=gen, device=dev).clamp_(max=1 - 2 ** -24)
    uni_t = torch.rand(B, Q, generator=gen, device=dev).clamp_(max=1 - 2 ** -24)
    seq = torch.empty((B, Q), dtype=torch.int32, device=dev)
    step_logits = torch.empty((B, V), dtype=torch.float32, device=dev)
    draft_logits = torch.empty((B, gamma, V), dtype=torch.float32, device=dev)
    logits = torch.empty((B * Q, V), dtype=torch.float32, device=dev)
    xd = torch.empty((B, 1, drf.shape.hidden), dtype=torch.bfloat16, device=dev)
    xt = torch.empty((B, Q, tgt.shape.hidden), dtype=torch.bfloat16, device=dev)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    out_tok = torch.empty((B, Q), dtype=torch.int32, device=dev)
    n0 = torch.empty((B,), dtype=torch.int32, device=dev)
    tok = torch.empty((B, 1), dtype=torch.int32, device=dev)
    ws = binding.workspace(1 << 28, dev)

    def draft_steps():
        seq[:, 0] = last
        for i in range(gamma):
            binding.embed_tokens(drf.table, seq[:, i].contiguous(), x=xd.view(B, -1))
            binding.verify_layers(drf.cfg, drf.stack, xd, pos_d[i], kv_d[i], l_max, ws=ws)
            if T == 0:      # arg-max straight out of the vocabulary projection, no logits written
                binding.lm_head_greedy_accept(xd, drf.final_norm, drf.w_lm, None, drf.shape.norm_eps, n_accepted=n0,
                                              out_tokens=tok, ws=ws)
            else:
                binding.lm_head_logits(xd.view(B, -1), drf.final_norm, drf.w_lm, drf.shape.norm_eps, out=step_logits, ws=ws)
                binding.spec_accept(step_logits.view(B, 1, V), None, None, uni_d[i], T, n_accepted=n0, out_tokens=tok, ws=ws)
                draft_logits[:, i].copy_(step_logits)
            seq[:, i + 1] = tok[:, 0]

    def verify():
        binding.embed_tokens(tgt.table, seq.view(-1), x=xt.view(B * Q, -1))
        binding.verify_layers(tgt.cfg, tgt.stack, xt, pos_t, kv_t, l_max, ws=ws)
        if T == 0:
            binding.lm_head_greedy_accept(xt, tgt.final_norm, tgt.w_lm, seq[:, 1:].contiguous(), tgt.shape.norm_eps,
                                          n_accepted=n_acc, out_tokens=out_tok, ws=ws)
        else:
            binding.lm_head_logits(xt.view(B * Q, -1), tgt.final_norm, tgt.w_lm, tgt.shape.norm_eps, out=logits, ws=ws)
            binding.spec_accept(logits.view(B, Q, V), draft_logits, seq[:, 1:].contiguous(), uni_t, T,
                                n_accepted=n_acc, out_tokens=out_tok, ws=ws)

    def timed(fn, iters):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters

    for _ in range(args.warmup):
        draft_steps(); verify()
    it_ms = timed(lambda: (draft_steps(), verify()), args.steps)
    d_ms = timed(draft_steps, args.steps)
    v_ms = timed(verify, args.steps)
    emitted = int((n_acc + 1).sum().item())
    return {
        "metric": "whole speculative-decoding iteration (drafting loop + verify step)", "unit": "tokens/s",
        "value": round(emitted / (it_ms * 1e-3), 1), "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(it_ms, 4), "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "7B-shaped target + 1.5B-shaped drafter, %d layers each, B=8, gamma=5, "
                               "kv_len U[1024,2048], T=%g" % (n_layers, T)},
        "draft_loop_ms": round(d_ms, 4), "draft_step_ms": round(d_ms / gamma, 4), "verify_ms": round(v_ms, 4),
        "cost_ratio_draft_step_over_verify": round(d_ms / gamma / v_ms, 4),
        "draft_step_weight_stream_GBps": round(drf.weight_bytes / (d_ms / gamma * 1e-3) / 1e9, 1),
        "verify_weight_stream_GBps": round(tgt.weight_bytes / (v_ms * 1e-3) / 1e9, 1),
        "mean_emitted_per_sequence": round(emitted / B, 3),
    }


def time_calls(torch, fn, iters=100, warm=10, stats=None):
    """Mean time per call (ms) of `iters` back-to-back calls after `warm` warm-ups; with `stats` (a dict) also the
    median, 10th and 90th percentile (us) of the same calls timed one by one with their own event pairs."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    mean_ms = a.elapsed_time(b) / iters
    if stats is not None:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for e0, e1 in evs:
            e0.record(); fn(); e1.record()
        torch.cuda.synchronize()
        t = np.sort(np.array([e0.elapsed_time(e1) for e0, e1 in evs])) * 1e3
        stats.update(median_us=round(float(np.median(t)), 1), p10_us=round(float(t[int(0.1 * iters)]), 1),
                     p90_us=round(float(t[int(0.9 * iters)]), 1), calls=iters)
    return mean_ms


def linear_prefill(torch, binding, synth, dev, gen):
    """Compute-bound counterpart of the verify projections: 4096 rows (an image-prefill-sized batch) through the
    3584 -> 18944 gate projection.  Run before the long memory-bound sections: a matrix-bound kernel is the one most
    sensitive to the clock the part sustains, and after seconds of full-bandwidth streaming the same launch is
    20-25 % slower."""
    s = synth.QWEN7B
    bf = torch.bfloat16
    Ml, Nl, Kl = 4096, s.mlp, s.hidden
    xl = torch.randn(Ml, Kl, generator=gen, device=dev).to(bf)
    wl = binding.weight_pack((torch.randn(Nl, Kl, generator=gen, device=dev) * 0.02).to(bf))
    yl = torch.empty((Ml, Nl), dtype=bf, device=dev)
    st = {}
    lin_ms = time_calls(torch, lambda: binding.linear(xl, wl, out=yl), 20, 5, stats=st)
    lin_flops = 2.0 * Ml * Nl * Kl
    t = st["median_us"] * 1e-6
    return {"shape": "M=4096, K=3584, N=18944 bf16", "bound": "mfma", "flops": lin_flops,
            "call_us": st["median_us"], "p10_us": st["p10_us"], "p90_us": st["p90_us"], "mean_back_to_back_us": round(lin_ms * 1e3, 1),
            "what": "whole call: operand re-layout kernel (about 25 us) + tile kernel",
            "TFLOPs": round(lin_flops / t / 1e12, 1), "peak_TFLOPs": 2500.0, "frac_of_bf16_peak": round(lin_flops / t / 2.5e15, 4)}


def prefill_attention_bench(torch, binding, synth, dev, gen):
    """Prompt-pass attention (compute-bound): 8 fresh prompts of 2048 positions (1280 image rows first), 28/4 heads,
    d=128, causal.  Flops = 4 d n_q sum_i (visible keys of position i)."""
    s = synth.QWEN7B
    bf = torch.bfloat16
    B, L = 8, 2048
    q = torch.randn(B, L, s.n_q_heads, s.head_dim, generator=gen, device=dev).to(bf)
    k = binding.k_cache_pack(torch.randn(B, s.n_kv_heads, L, s.head_dim, generator=gen, device=dev).to(bf))
    v = binding.v_cache_pack(torch.randn(B, s.n_kv_heads, L, s.head_dim, generator=gen, device=dev).to(bf))
    zero = torch.zeros(B, dtype=torch.int32, device=dev)
    n_new = torch.full((B,), L, dtype=torch.int32, device=dev)
    out = torch.empty_like(q)
    st = {}
    mean_ms = time_calls(torch, lambda: binding.prefill_attention(q, k, v, zero, n_new, out=out), 20, 5, stats=st)
    flops = 4.0 * s.head_dim * s.n_q_heads * B * (L * (L + 1) / 2)
    t = st["median_us"] * 1e-6
    return {"shape": f"B={B}, {L} new positions each (fresh prompt), 28/4 heads, d=128, causal, bf16", "bound": "mfma",
            "flops": flops, "call_us": st["median_us"], "p10_us": st["p10_us"], "p90_us": st["p90_us"],
            "mean_back_to_back_us": round(mean_ms * 1e3, 1), "TFLOPs": round(flops / t / 1e12, 1),
            "peak_TFLOPs": 2500.0, "frac_of_bf16_peak": round(flops / t / 2.5e15, 4)}


def extra_bandwidth(torch, binding, synth, dev, gen):
    """Second half of the metric: HBM GB/s of verify_attention and spec_accept at the long-context
    batched shape (B=32, gamma=7, KV 8192 bf16, 28/4 heads, d=128, V=152064, T=0.7).  Several
    buffer sets are rotated so that the 256 MB last-level cache cannot serve the stream."""
    s = synth.QWEN7B
    B, gamma, L, V = 32, 7, 8192, s.vocab
    Q = gamma + 1
    l_max = (L + Q + 31) // 32 * 32
    bf = torch.bfloat16
    sets = 3
    qs = [torch.randn(B, Q, s.n_q_heads, s.head_dim, generator=gen, device=dev).to(bf) for _ in range(sets)]
    ks = [binding.k_cache_pack(torch.randn(B, s.n_kv_heads, l_max, s.head_dim, generator=gen, device=dev).to(bf)) for _ in range(sets)]
    vs = [binding.v_cache_pack(torch.randn(B, s.n_kv_heads, l_max, s.head_dim, generator=gen, device=dev).to(bf))
          for _ in range(sets)]
    kv_len = torch.full((B,), L, dtype=torch.int32, device=dev)
    out = torch.empty_like(qs[0])
    it = [0]

    def attn():
        i = it[0] % sets
        it[0] += 1
        binding.verify_attention(qs[i], ks[i], vs[i], kv_len, out=out)

    attn_stats, acc_stats, acc0_stats = {}, {}, {}
    attn_ms = time_calls(torch, attn, stats=attn_stats)
    attn_bytes = B * 2 * (L + Q) * s.n_kv_heads * s.head_dim * 2
    del qs, ks, vs

    T = float(np.float32(0.7))
    tls, dls = [], []
    for _ in range(2):
        t = torch.randn(B, Q, V, generator=gen, device=dev) * 3.0
        dl = 0.8 * t[:, :gamma] + 0.6 * 3.0 * torch.randn(B, gamma, V, generator=gen, device=dev)
        tls.append(t.contiguous()); dls.append(dl.contiguous())
    toks = dls[0].argmax(-1).to(torch.int32)
    u = torch.rand(B, Q, generator=gen, device=dev).clamp_(max=1 - 2 ** -24)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    out_tok = torch.empty((B, Q), dtype=torch.int32, device=dev)

    def acc_t():
        i = it[0] % 2
        it[0] += 1
        binding.spec_accept(tls[i], dls[i], toks, u, T, n_accepted=n_acc, out_tokens=out_tok)

    def acc_0():
        i = it[0] % 2
        it[0] += 1
        binding.spec_accept(tls[i], None, toks, None, 0.0, n_accepted=n_acc, out_tokens=out_tok)

    acc_ms = time_calls(torch, acc_t, stats=acc_stats)
    acc0_ms = time_calls(torch, acc_0, stats=acc0_stats)
    acc_bytes = B * Q * V * 4 + B * gamma * V * 4 + B * 2 * V * 4
    acc0_bytes = B * Q * V * 4
    gb = lambda nbytes, ms: round(nbytes / (ms * 1e-3) / 1e9, 1)
    del tls, dls

    # a plain device copy in the same run: the bandwidth a trivial kernel reaches on this machine (read + write bytes)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    copy_ms = time_calls(torch, lambda: dst.copy_(src), 10, 3)
    copy_gbps = round(2 * src.numel() / (copy_ms * 1e-3) / 1e9, 1)
    del src, dst

    def entry(nbytes, mean_ms, st):
        # bandwidth from the median of the singly timed calls (the back-to-back mean also contains the host's
        # launch rate: one Python call per ~100 us of GPU work)
        g = gb(nbytes, st["median_us"] * 1e-3)
        return {"us": st["median_us"], "GBps": g, "frac_of_8TBps": round(g / HBM_PEAK_GBS, 4),
                "frac_of_device_copy": round(g / copy_gbps, 4), "bytes": nbytes, "p10_us": st["p10_us"],
                "p90_us": st["p90_us"], "mean_back_to_back_us": round(mean_ms * 1e3, 1), "calls": st["calls"]}

    return {
        "workload": "long-context batched: B=32, gamma=7, KV 8192 bf16, 28/4 heads, d=128, V=152064",
        "timing": "us = median of 100 calls timed singly with HIP events after 10 warm-ups (p10 / p90 beside it; also the mean of 100 back-to-back calls); "
                  "3 (attention) and 2 (accept) rotating input sets of 540 / 290 MB each, larger than the 256 MB last-level cache",
        "device_copy_GBps": copy_gbps,
        "verify_attention": entry(attn_bytes, attn_ms, attn_stats),
        "spec_accept_T0.7": entry(acc_bytes, acc_ms, acc_stats),
        "spec_accept_T0": entry(acc0_bytes, acc0_ms, acc0_stats),
    }


def cpu_legs(torch, binding, wl, shape, cfg, raw0, layer0, x0, x_final, pos, kv_len, kv_len_h, l_max,
             final_norm, w_lm_rows, logits, draft_logits, draft_tokens, uniforms, n_acc, out_tok, T, ws):
    """The CPU checker on the very tensors the timed step ran on (downloaded from the device), outside the timed
    region.  Returns (parity, cpu_baseline).

    parity: layer 0 (the timed stack's first layer, re-run alone on the step's input x0; the cache rows the timed
    run itself appended in layer 0), the vocabulary projection (the timed run's final hidden rows -> its logits) and
    the accept rule (the timed run's logits and drafts -> its n_accepted / out_tokens).  The 27 layers between are
    covered by the chain test, not here: the checker would need every layer's weights on the host.
    cpu_baseline: the same checker calls timed -- pinned to one thread, then with all cores -- on a bounded sample:
    one layer pass (single thread) / layer passes until ~10 s (all cores) with layer 0's weights, scaled by the
    layer count, + the vocabulary projection + the accept rule."""
    from oracle import verify_oracle as O
    from threadpoolctl import threadpool_limits, threadpool_info
    B, gamma, N = wl["batch"], wl["gamma"], wl["layers"]
    Q = gamma + 1
    f32 = lambda t: t.float().cpu().numpy()
    rel = lambda g, r: float(np.max(np.abs(np.asarray(g, np.float64) - r)) / max(np.max(np.abs(r)), 1e-30))
    cores = len(os.sched_getaffinity(0))
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass

    # ---- layer 0 ----
    w = {k: (None if v is None else f32(v)) for k, v in raw0["w"].items()}
    xh, kh, vh, posh = f32(x0), f32(raw0["k"]), f32(raw0["v"]), pos.cpu().numpy()
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        y_ref, k_ref, v_ref = O.verify_layer(shape, w, xh, posh, kh, vh, kv_len_h)
        t_layer_1 = time.perf_counter() - t0
    x1 = x0.clone()
    stack1 = binding.LayerStack([layer0[1]], [layer0[2]], [layer0[3]])
    desc1 = binding.layer_desc(cfg, B, Q, l_max, binding.BF16)
    binding.verify_layers(cfg, stack1, x1, pos, kv_len, l_max, ws=ws, desc=desc1)
    torch.cuda.synchronize()
    e_layer = rel(f32(x1), y_ref)
    # cache rows appended by the timed run (library layouts -> rows)
    nkv, d = shape.n_kv_heads, shape.head_dim
    k_rows = layer0[2].reshape(B, nkv, l_max // 32, 2, d // 8, 4, 4, 8).permute(0, 1, 2, 5, 3, 6, 4, 7).reshape(B, nkv, l_max, d)
    v_rows = layer0[3].permute(0, 1, 2, 4, 3).reshape(B, nkv, l_max, d)
    kg, vg = f32(k_rows), f32(v_rows)
    e_k = max(rel(kg[b, :, L:L + Q], k_ref[b, :, L:L + Q]) for b, L in enumerate(int(v) for v in kv_len_h))
    e_v = max(rel(vg[b, :, L:L + Q], v_ref[b, :, L:L + Q]) for b, L in enumerate(int(v) for v in kv_len_h))
    # all cores: passes with the same weights until ~10 s have gone by
    t_layers, passes, y = 0.0, 0, xh
    while passes < N and t_layers < 10.0:
        t0 = time.perf_counter()
        y, _, _ = O.verify_layer(shape, w, y, posh, kh, vh, kv_len_h)
        t_layers += time.perf_counter() - t0
        passes += 1
    t_layer_n = t_layers / passes
    del w, kh, vh, kg, vg

    # ---- vocabulary projection on the timed run's final hidden rows ----
    xf, gn, wl_h = f32(x_final).reshape(B * Q, -1), f32(final_norm), f32(w_lm_rows)
    t0 = time.perf_counter()
    logits_ref = O.lm_head_logits(xf, gn, wl_h, shape.norm_eps)
    t_lm_n = time.perf_counter() - t0
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        O.lm_head_logits(xf, gn, wl_h, shape.norm_eps)
        t_lm_1 = time.perf_counter() - t0
    del wl_h
    lg = logits.cpu().numpy()
    e_logits = rel(lg, logits_ref)
    del logits_ref

    # ---- accept rule on the timed run's own logits ----
    tl = lg.reshape(B, Q, -1)
    dl = draft_logits.cpu().numpy() if T > 0 else None
    u = uniforms.cpu().numpy() if T > 0 else None
    t0 = time.perf_counter()
    n_ref, out_ref, margin = O.spec_accept(tl, dl, draft_tokens.cpu().numpy(), u, T)
    t_acc = time.perf_counter() - t0
    n_g, out_g = n_acc.cpu().numpy(), out_tok.cpu().numpy()
    clear = bool(np.all(margin > 1e-5))
    parity = {"what": "CPU checker on the tensors of the timed run: layer 0 re-run alone on the step's input, the cache "
                      "rows the timed run appended in layer 0, its logits from its final hidden rows, its accept outputs "
                      "from its logits",
              "layer0_max_rel_err": round(e_layer, 5), "appended_k_max_rel_err": round(e_k, 5),
              "appended_v_max_rel_err": round(e_v, 5), "logits_max_rel_err": round(e_logits, 5), "bound": 2e-2,
              "n_accepted_equal": bool(np.array_equal(n_g, n_ref)), "out_tokens_equal": bool(np.array_equal(out_g, out_ref)),
              "decision_margins_clear": clear,
              "ok": bool(max(e_layer, e_k, e_v, e_logits) <= 2e-2 and np.array_equal(n_g, n_ref) and
                         (np.array_equal(out_g, out_ref) or not clear))}
    emitted = float((n_ref + 1).sum())
    t_step_n = N * t_layer_n + t_lm_n + t_acc
    t_step_1 = N * t_layer_1 + t_lm_1 + t_acc
    blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    cpu = {"value": round(emitted / t_step_n, 3), "unit": "tokens/s", "cores": int(min(cores, blas)), "kind": "oracle",
           "sample": f"all cores: {passes} of {N} layer passes (all {B} sequences, layer 0's weights) timed {t_layers:.2f}s, "
                     f"mean scaled x{N}, + lm_head {t_lm_n:.2f}s + accept {t_acc:.2f}s; float64 NumPy on the timed run's tensors",
           "est_ms_per_step": round(t_step_n * 1e3, 1),
           "single_thread": {"value": round(emitted / t_step_1, 4), "cores": 1, "est_ms_per_step": round(t_step_1 * 1e3, 1),
                             "sample": f"1 layer pass {t_layer_1:.2f}s scaled x{N} + lm_head {t_lm_1:.2f}s + accept {t_acc:.2f}s"},
           "affinity_cores": cores, "cpu_model": cpu_model}
    return parity, cpu


if __name__ == "__main__":
    main()
