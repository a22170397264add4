"""Benchmark of the layer training step (forward + backward) on one MI355X.

One "step" = slapo_layer_fwd + slapo_layer_bwd over one synthetic batch that already sits in HBM.
Prints ONE JSON line: whole-job samples/s plus the roofline record of the dominant kernel (measured
live with HIP events on the launch stream) and the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

import workloads as W

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (figures and commands in profiles/); None where no counter run has been made.
TRAFFIC_BYTES_PER_LAUNCH = {"C2-bert-large-layer-bf16": 108.49e6}   # 100.80 MB fetched + 7.69 MB written


def layer_flops(cfg, seqlens):
    """Algorithmic FLOPs of one layer forward+backward: 3 x GEMM + 3.5 x visible attention."""
    T, H, F, S = cfg.tokens, cfg.hidden, cfg.ffn, cfg.seq
    gemm_fwd = 2.0 * T * (4.0 * H * cfg.attn_width + (3.0 if cfg.arch == W.LLAMA else 2.0) * H * F)   # gated FFN: three F x H products
    lens = [S] * cfg.batch if seqlens is None else [int(v) for v in seqlens]
    phi = 0.5 * (1.0 + 1.0 / S) if cfg.causal else 1.0
    att_fwd = sum(4.0 * cfg.attn_width * S * l * phi for l in lens)
    return 3.0 * gemm_fwd + 3.5 * att_fwd, gemm_fwd, att_fwd


def event_time_ms(fn, iters, stream):
    """Average duration of fn() over `iters` launches, HIP events recorded on the launch stream."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(iters):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def torch_eager_step_ms(cfg, params, x, dy, seqlens, iters, stream):
    """Context only: the same layer as an unfused chain of PyTorch library ops with autograd on the same GPU
    (vendor GEMMs, the framework's attention, dropout, normalisation and activation kernels), the kind of
    execution the paper's schedules start from. Returns milliseconds per forward+backward."""
    import torch.nn.functional as F
    dev = "cuda"
    tdt = {W.FP32: torch.float32, W.FP16: torch.float16}.get(cfg.dtype, torch.bfloat16)
    P = {k: torch.from_numpy(v).to(dev).to(tdt).requires_grad_(True) for k, v in params.items()}
    xt = torch.from_numpy(x).to(dev).to(tdt).requires_grad_(True)
    dyt = torch.from_numpy(dy).to(dev).to(tdt)
    B_, S, H, h = cfg.batch, cfg.seq, cfg.hidden, cfg.heads
    d = H // h
    mask = None
    if seqlens is not None:
        mask = (torch.arange(S, device=dev)[None, :] < torch.from_numpy(seqlens).to(dev)[:, None])[:, None, None, :]
        if cfg.causal:
            mask = mask & torch.tril(torch.ones(S, S, dtype=torch.bool, device=dev))[None, None]
    llama = cfg.arch == W.LLAMA
    if llama:
        inv = 1.0 / (cfg.rope_base ** (torch.arange(0, d, 2, device=dev, dtype=torch.float32) / d))
        ang = torch.outer(torch.arange(S, device=dev, dtype=torch.float32), inv)
        cos, sin = ang.cos().to(tdt)[None, :, None, :], ang.sin().to(tdt)[None, :, None, :]

        def rot(t):   # [B,S,h,d], adjacent pairs
            e, o = t[..., 0::2], t[..., 1::2]
            return torch.stack((e * cos - o * sin, e * sin + o * cos), dim=-1).reshape(t.shape)

    def norm(t, k):
        if llama:
            return F.rms_norm(t, (H,), P[k + "_g"], cfg.ln_eps)
        return F.layer_norm(t, (H,), P[k + "_g"], P[k + "_b"], cfg.ln_eps)

    def layer(t):
        a_in = norm(t, "ln1") if cfg.pre_ln else t
        q, k, v = F.linear(a_in, P["wqkv"], P.get("bqkv")).split(H, dim=-1)
        q, k, v = (u.reshape(B_, S, h, d) for u in (q, k, v))
        if llama:
            q, k = rot(q), rot(k)
        q, k, v = (u.transpose(1, 2) for u in (q, k, v))
        a = F.scaled_dot_product_attention(q, k, v, attn_mask=mask, dropout_p=cfg.attn_dropout_p,
                                           is_causal=bool(cfg.causal) and mask is None)
        a = a.transpose(1, 2).reshape(B_, S, H)
        z1 = t + F.dropout(F.linear(a, P["wo"], P.get("bo")), cfg.dropout_p)
        f_in = norm(z1, "ln2") if cfg.pre_ln else norm(z1, "ln1")
        if llama:
            uv = F.linear(f_in, P["w1"])
            g = F.silu(uv[..., 0::2]) * uv[..., 1::2]
        else:
            u = F.linear(f_in, P["w1"], P["b1"])
            g = F.gelu(u) if cfg.act == W.GELU else F.relu(u)
        r2 = F.dropout(F.linear(g, P["w2"], P.get("b2")), cfg.dropout_p)
        return z1 + r2 if cfg.pre_ln else norm(f_in + r2, "ln2")

    def step():
        for t in P.values():
            t.grad = None
        xt.grad = None
        layer(xt).backward(dyt)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    return event_time_ms(step, iters, stream)


def cpu_baseline(cfg, params, x, dy, seqlens):
    """The fp64 oracle, as it stands, on the host cores: one full layer forward+backward."""
    if cfg.arch == W.LLAMA:
        from oracle import llama_layer as L
    else:
        from oracle import layer as L
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    reps, t0 = 0, time.perf_counter()
    while True:   # whole layers until about ten seconds of CPU work are on the clock
        c = L.layer_forward(cfg, params, x, seqlens)
        L.layer_backward(cfg, params, c, dy)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 64:
            break
    return {"value": reps * cfg.batch / dt, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} x one full {cfg.name} layer forward+backward (batch {cfg.batch}), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "C6"],
                    help="C5 = the 24-layer stack (one step = 24 layer forwards, then 24 layer backwards); "
                         "C6 = the LLaMA-7B-shaped layer (RMSNorm, rotary, SwiGLU)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--checkpoint", action="store_true",
                    help="activation-checkpointing mode: nothing saved, backward recomputes the forward")
    ap.add_argument("--fp16", action="store_true", help="IEEE half storage instead of bf16 (same kernels)")
    ap.add_argument("--attn-dropout", type=float, default=0.0,
                    help="also drop attention probabilities with this probability (0 = the benchmark configuration)")
    ap.add_argument("--breakdown", action="store_true", help="also time each GEMM / kernel class (stderr)")
    ap.add_argument("--layers", type=int, default=0,
                    help="run the configuration as a stack of this many layers (default: the configuration's own count)")
    ap.add_argument("--tp", type=int, default=1,
                    help="time ONE rank's share of the layer sharded N ways along heads and FFN columns "
                         "(heads/N, attention width hidden/N, ffn/N; no collectives are run)")
    ap.add_argument("--eager-baseline", action="store_true",
                    help="also time the same layer as unfused PyTorch library ops with autograd (context, in `extra`)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU sharding is design-only.",
              file=sys.stderr)
        sys.exit(2)

    from paper_2302_08005_amd import binding as B

    cfg = W.CONFIGS[args.config]
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    if args.attn_dropout:
        cfg = cfg.replace(attn_dropout_p=args.attn_dropout)
    if args.fp16:
        cfg = cfg.replace(dtype=W.FP16)
    if args.layers > 0 and args.layers != cfg.n_layers:
        cfg = cfg.replace(name=f"{cfg.name}-x{args.layers}", n_layers=args.layers)
    if args.tp > 1:
        if cfg.heads % args.tp or cfg.ffn % (8 * args.tp):
            sys.exit(f"bench.py: --tp {args.tp} does not divide {cfg.heads} heads / ffn {cfg.ffn}")
        cfg = cfg.replace(name=f"{cfg.name}-tp{args.tp}-share", heads=cfg.heads // args.tp, attn_dim=cfg.hidden // args.tp,
                          ffn=cfg.ffn // args.tp)
    params = W.make_params(cfg)
    x, dy, seqlens = W.make_inputs(cfg)
    layer = B.Layer(cfg, params, checkpoint=1 if args.checkpoint else 0)
    xd, dyd = layer.to_device(x), layer.to_device(dy)
    sld = None if seqlens is None else torch.from_numpy(seqlens).cuda()
    y = torch.empty_like(xd)
    dx = torch.empty_like(xd)

    def step():
        B.slapo_layer_fwd(layer.desc, layer.params, xd, sld, y, layer.saved, layer.scratch)
        B.slapo_layer_bwd(layer.desc, layer.params, xd, sld, dyd, layer.saved, dx, layer.grads, layer.scratch)

    if cfg.n_layers > 1:   # the stack: per-layer weights seeded by the layer index, dy injected at the top
        stack = B.Stack(cfg, [W.make_params(cfg, layer_id=l) for l in range(cfg.n_layers)],
                        checkpoint=1 if args.checkpoint else 0)

        def step():
            B.slapo_stack_fwd(stack.desc, stack.params, xd, sld, y, stack.acts, stack.saved, stack.scratch)
            B.slapo_stack_bwd(stack.desc, stack.params, xd, sld, dyd, stack.acts, stack.saved, dx, stack.grads,
                              stack.scratch)

    if args.calibrate_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    gpu_ms = e0.elapsed_time(e1) / args.steps
    ms = max(wall_ms, gpu_ms)

    total_flops, gemm_fwd, att_fwd = layer_flops(cfg, seqlens)
    total_flops *= cfg.n_layers
    T, H, F = cfg.tokens, cfg.hidden, cfg.ffn
    dt, act = cfg.dtype, cfg.act

    # Dominant kernel: the weight-gradient (TN) GEMM kernel. One kernel symbol serves dW2 = dR2^T G,
    # dW1 = dU^T Y1 and dWqkv = dQKV^T X (three launches per step, the largest share of the step in the
    # rocprofv3 trace). The three launches are repeated here exactly as the layer issues them (same shapes,
    # same tile selection), alone on the launch stream between HIP events.
    tdt = xd.dtype
    mk = lambda *shape: torch.randn(*shape, device="cuda", dtype=torch.float32).to(tdt)
    llama = cfg.arch == W.LLAMA
    F1 = 2 * F if llama else F                                  # rows of w1 (gate and up rows interleaved)
    tn_shapes = [(H, F, T), (F1, H, T), (3 * cfg.attn_width, H, T)]   # (M, N, K): C[M,N] = A[K,M]^T B[K,N]
    tn_bufs = [(mk(K, M), mk(K, N), torch.empty(M, N, device="cuda", dtype=tdt)) for (M, N, K) in tn_shapes]

    def dominant():
        for (M, N, K), (a, b, c) in zip(tn_shapes, tn_bufs):
            B.slapo_gemm(dt, B.TN, B.EPI_NONE, act, M, N, K, a, b, c)

    for _ in range(5):
        dominant()
    reps = max(20, args.steps)
    dom_ms = event_time_ms(dominant, reps, stream) / len(tn_shapes)      # average per launch
    dom_flops = sum(2.0 * M * N * K for (M, N, K) in tn_shapes) / len(tn_shapes)
    achieved = dom_flops / (dom_ms * 1e-3) / 1e12
    tile = "128,128,64" if cfg.name.startswith("C2") else "..."   # (tile choice depends on the shape; C2's is the profiled one)
    roofline = {"bound": "mfma", "kernel": f"gemm_bf16_kernel<TN,{tile},...> (weight gradients dW2, dW1, dWqkv)",
                "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(cfg.name),
                "avg_launch_us": dom_ms * 1e3, "flop_per_launch": dom_flops}

    if args.checkpoint:   # the isolated-kernel figures below read saved activations: take them from a plain layer
        layer = B.Layer(cfg, params)
    if args.checkpoint or cfg.n_layers > 1:
        B.slapo_layer_fwd(layer.desc, layer.params, xd, sld, y, layer.saved, layer.scratch)
        torch.cuda.synchronize()
    # for reference: the largest forward GEMM with its fused bias+activation epilogue (FFN1)
    y1 = layer.saved_tensor("n2" if cfg.pre_ln else "y1")
    # (a ReLU layer keeps no derivative: its gate is read off the activation output)
    u = layer.saved_tensor("dgate") if llama else layer.saved_tensor("dact") if act == W.GELU else None
    g = torch.empty(T * F, device="cuda", dtype=tdt)

    def ffn1():
        if llama:
            B.slapo_gemm(dt, B.NT, B.EPI_GATE, act, T, 2 * F, H, y1, layer.params["w1"], g, aux_out=u)
        else:
            B.slapo_gemm(dt, B.NT, B.EPI_BIAS_ACT, act, T, F, H, y1, layer.params["w1"], g, bias=layer.params["b1"], aux_out=u)

    for _ in range(5):
        ffn1()
    ffn1_ms = event_time_ms(ffn1, reps, stream)
    ffn1_tf = 2.0 * T * F1 * H / (ffn1_ms * 1e-3) / 1e12

    # the HBM-bound fused epilogue (bias+dropout+residual+LayerNorm forward), algorithmic bytes 4*T*H*eb
    eb = 4 if cfg.dtype == W.FP32 else 2
    r = torch.empty_like(xd).view(T, H)
    z = torch.empty_like(r)
    o = torch.empty_like(r)
    mu = torch.empty(T, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mu)

    def epi():
        B.slapo_bdrln_fwd(layer.desc, 0, T, r, layer.params.get("bo"), xd, layer.params["ln1_g"], layer.params.get("ln1_b"), z, o, mu, rstd)

    r.normal_()
    for _ in range(5):
        epi()
    epi_ms = event_time_ms(epi, max(20, args.steps), stream)
    epi_gbs = 4.0 * T * H * eb / (epi_ms * 1e-3) / 1e9

    # context for "achievable" HBM bandwidth: a plain device-to-device copy of 256 MiB (read + write counted)
    csrc = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    cdst = torch.empty_like(csrc)
    for _ in range(3):
        cdst.copy_(csrc)
    copy_ms = event_time_ms(lambda: cdst.copy_(csrc), 20, stream)
    copy_gbs = 2.0 * (256 << 20) / (copy_ms * 1e-3) / 1e9
    del csrc, cdst

    extra = {"copy_kernel_256MiB": {"achieved": copy_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": copy_gbs / HBM_PEAK_GBS},
             "ffn1_fwd_gemm_bias_act": {"bound": "mfma", "achieved": ffn1_tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                                        "unit": "TFLOP/s", "frac": ffn1_tf / MFMA_BF16_PEAK_TFLOPS,
                                        "avg_launch_us": ffn1_ms * 1e3},
             "layer_tflops": total_flops / (ms * 1e-3) / 1e12,
             "layer_frac_of_mfma_peak": total_flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
             "gpu_event_ms_per_step": gpu_ms, "wall_ms_per_step": wall_ms,
             "epilogue_bdrln_fwd": {"bound": "hbm", "achieved": epi_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": epi_gbs / HBM_PEAK_GBS, "avg_launch_us": epi_ms * 1e3}}

    if args.breakdown:
        breakdown(cfg, layer, xd, dyd, sld, stream)
    if args.eager_baseline and cfg.n_layers == 1:
        eager_ms = torch_eager_step_ms(cfg, params, x, dy, seqlens, max(10, args.steps // 2), stream)
        extra["torch_eager_unfused"] = {"ms_per_step": eager_ms, "speedup_of_this_library": eager_ms / ms}

    out = {"metric": "layer fwd+bwd samples/s", "value": cfg.batch / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": {W.BF16: "bf16", W.FP16: "f16"}.get(cfg.dtype, "f32"),
           "data": "synthetic",
           "config": {"workload": cfg.name, "batch": cfg.batch, "seq": cfg.seq, "hidden": cfg.hidden,
                      "heads": cfg.heads, "ffn": cfg.ffn, "causal": cfg.causal, "dropout_p": cfg.dropout_p,
                      "attn_dropout_p": cfg.attn_dropout_p, "pre_ln": cfg.pre_ln, "layers": cfg.n_layers, "checkpoint": int(args.checkpoint),
                      "family": "llama" if llama else "classic", "tp_share": args.tp,
                      "parallelism": "single-gpu"},
           "roofline": roofline, "extra": extra}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, params, x, dy, seqlens)
    print(json.dumps(out), flush=True)


def breakdown(cfg, layer, xd, dyd, sld, stream):
    """Per-GEMM timings through the exported building blocks (diagnostics on stderr)."""
    from paper_2302_08005_amd import binding as B
    T, H, F = cfg.tokens, cfg.hidden, cfg.ffn
    dt = cfg.dtype
    dev = xd.device
    tdt = xd.dtype
    mk = lambda *s: torch.randn(*s, device=dev, dtype=torch.float32).to(tdt)
    F1 = 2 * F if cfg.arch == W.LLAMA else F
    shapes = [("qkv  NT", B.NT, T, 3 * H, H), ("out  NT", B.NT, T, H, H), ("ffn1 NT", B.NT, T, F1, H), ("ffn2 NT", B.NT, T, H, F),
              ("dG   NN", B.NN, T, F, H), ("dY1  NN", B.NN, T, H, F1), ("dA   NN", B.NN, T, H, H), ("dX   NN", B.NN, T, H, 3 * H),
              ("dW2  TN", B.TN, H, F, T), ("dW1  TN", B.TN, F1, H, T), ("dWo  TN", B.TN, H, H, T), ("dWqkv TN", B.TN, 3 * H, H, T)]
    tot = 0.0
    for name, layout, M, N, K in shapes:
        a = mk(M, K) if layout != B.TN else mk(K, M)
        b = mk(N, K) if layout == B.NT else mk(K, N)
        c = torch.empty(M, N, device=dev, dtype=tdt)
        fn = lambda: B.slapo_gemm(dt, layout, B.EPI_NONE, 0, M, N, K, a, b, c)
        for _ in range(3):
            fn()
        ms = event_time_ms(fn, 20, stream)
        tot += ms
        print(f"  {name}: M={M} N={N} K={K}: {ms * 1e3:8.1f} us  {2.0 * M * N * K / ms / 1e9:8.1f} TFLOP/s", file=sys.stderr)
    print(f"  GEMM total {tot * 1e3:.1f} us", file=sys.stderr)
    desc = layer.desc
    qkv = layer.saved_tensor("qkv")
    attn = layer.saved_tensor("attn")
    lse = layer.saved_tensor("lse")
    out = torch.empty_like(attn)
    fn = lambda: B.slapo_attn_fwd(desc, qkv, sld, out, lse)
    fn()
    ms = event_time_ms(fn, 20, stream)
    print(f"  attn fwd: {ms * 1e3:8.1f} us", file=sys.stderr)
    delta = torch.empty_like(lse)
    dqkv = torch.empty_like(qkv)
    fn = lambda: B.slapo_attn_bwd(desc, qkv, sld, attn, dyd, lse, delta, dqkv)
    fn()
    ms = event_time_ms(fn, 20, stream)
    print(f"  attn bwd: {ms * 1e3:8.1f} us", file=sys.stderr)


if __name__ == "__main__":
    main()
