"""Benchmark of the layer training step (forward + backward) on one MI355X.

One "step" = slapo_layer_fwd + slapo_layer_bwd (for the 24-layer stack: slapo_stack_fwd + slapo_stack_bwd) over
one synthetic batch that already sits in HBM. Prints ONE JSON line: whole-job samples/s of the headline
configuration, the roofline record of its dominant kernel (measured live with HIP events on the launch stream),
the CPU oracle timed on the host cores, and under extra.configs the same step figures for the other benchmark
configurations (C3, C4, C5), each with
  - the whole step: ms, samples/s, algorithmic TFLOP/s and the fraction of the bf16 MFMA peak,
  - the GEMM + attention kernels alone: every one of the 12 GEMMs (with its fused epilogue and the tile
    selection the step uses) and the attention forward / backward launched in isolation; their summed time
    against the step's algorithmic GEMM + attention work is the joint MFMA fraction of the kernels' own time,
  - the HBM-bound fused row kernels (forward and backward) over a rotation of disjoint buffer sets of at least
    1 GiB in total, so that no launch finds its operands in the 256 MB last-level cache.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

import workloads as W

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16
HBM_PEAK_GBS = 8000.0
ROTATE_BYTES = 1 << 30           # the HBM-bound loops walk through at least this much memory before reusing any
# HBM-side bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (figures, scale factors and commands in profiles/), keyed by workload and kernel instance; None where
# no counter run covers the pair.
TRAFFIC_BYTES_PER_LAUNCH = {
    # profiles/layer_step_C2_bert_large_hbm_traffic.txt: 100.77 MB fetched + 7.69 MB written
    ("C2-bert-large-layer-bf16", "gemm_bf16_kernel<2, 128, 128, 64, 2, 2, 2, 2, 4, 4, false, 0, false, false>"): 108.46e6,
    # profiles/layer_step_C4_gptneo_2p7b_hbm_traffic.txt: 819.48 MB fetched + 52.43 MB written
    ("C4-gptneo-2.7b-layer-bf16", "gemm_bf16_kernel<2, 256, 256, 64, 2, 4, 1, 2, 2, 0, false, 0, false, false>"): 871.91e6,
}


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


def timed(fn, iters, stream, warm=3):
    for _ in range(warm):
        fn()
    return event_time_ms(fn, iters, stream)


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


def kernel_figures(B, cfg, layer, xd, dyd, sld, seqlens, reps, stream, verbose=False):
    """Every GEMM and attention kernel of one layer step launched alone (fused epilogues and tile selection as in the
    step), the dominant kernel's roofline record, and the HBM-bound row kernels over rotating buffers."""
    T, H, F, A = cfg.tokens, cfg.hidden, cfg.ffn, cfg.attn_width
    dt, act, tdt = cfg.dtype, cfg.act, xd.dtype
    llama = cfg.arch == W.LLAMA
    F1 = 2 * F if llama else F
    post = not cfg.pre_ln
    P = layer.params

    def rnd(*shape):
        return torch.randn(*shape, device="cuda", dtype=torch.float32).mul_(0.5).to(tdt)

    B.slapo_layer_fwd(layer.desc, P, xd, sld, torch.empty_like(xd), layer.saved, layer.scratch)   # real activations in `saved`
    torch.cuda.synchronize()
    qkv, attn, lse, g = (layer.saved_tensor(k) for k in ("qkv", "attn", "lse", "g"))
    n_in = layer.saved_tensor("n2" if cfg.pre_ln else "y1")
    u = layer.saved_tensor("dgate") if llama else layer.saved_tensor("dact") if act == W.GELU else None
    th, tf, ta, t3a = rnd(T, H), rnd(T, F1), rnd(T, A), rnd(T, 3 * A)
    oth, otf, ota, ot3a, og = (torch.empty(T, n, device="cuda", dtype=tdt) for n in (H, F1, A, 3 * A, F))
    res = rnd(T, H)

    rows = []   # (name, algorithmic flop, fn, kernel instance)

    def gemm(name, shared, layout, epi, M, N, K, a, b, c, **kw):
        flags = B.GEMM_SHARED if shared else 0
        nbytes = B.slapo_gemm_workspace(dt, layout, epi, M, N, K)   # (the layer hands its GEMMs a region of its scratch)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
        rows.append((name, 2.0 * M * N * K, lambda: B.slapo_gemm_ex(dt, layout, epi, act, M, N, K, a, b, c, flags=flags, ws=ws, **kw),
                     B.slapo_gemm_kernel_name(dt, layout, epi, M, N, K, flags=flags, with_ws=1)))

    def wgrad(name, M, N, K, a, b):
        nbytes = B.slapo_weight_grad_workspace(dt, M, N, K)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        c = torch.empty(M, N, device="cuda", dtype=tdt)
        rows.append((name, 2.0 * M * N * K, lambda: B.slapo_weight_grad(dt, 0, M, N, K, a, b, c, ws),
                     B.slapo_gemm_kernel_name(dt, B.TN, B.EPI_NONE, M, N, K, flags=B.GEMM_SHARED, weight_grad=1, with_ws=1)))

    # forward: the GEMM has the chip to itself
    if llama:
        gemm("qkv", False, B.NT, B.EPI_NONE, T, 3 * A, H, n_in, P["wqkv"], ot3a)
    else:
        gemm("qkv", False, B.NT, B.EPI_BIAS, T, 3 * A, H, n_in, P["wqkv"], ot3a, bias=P["bqkv"])
    gemm("out", False, B.NT, B.EPI_NONE, T, H, A, attn, P["wo"], oth)
    if llama:
        gemm("ffn1+gate", False, B.NT, B.EPI_GATE, T, 2 * F, H, n_in, P["w1"], og, aux_out=otf)
    else:
        gemm("ffn1+bias+act", False, B.NT, B.EPI_BIAS_ACT, T, F, H, n_in, P["w1"], og, bias=P["b1"],
             aux_out=(otf if act == W.GELU else None))
    gemm("ffn2", False, B.NT, B.EPI_NONE, T, H, F, g, P["w2"], oth)
    # backward: the data-gradient chain shares the chip with the weight gradients of the helper stream
    if llama:
        gemm("dG+dgate", True, B.NN, B.EPI_DGATE, T, F, H, th, P["w2"], otf, aux_in=u)
    else:
        gemm("dG+dact", True, B.NN, B.EPI_DACT, T, F, H, th, P["w2"], otf, aux_in=(u if u is not None else g))
    if post:
        gemm("dY1+add", True, B.NN, B.EPI_ADD, T, H, F1, tf, P["w1"], oth, aux_in=res)
    else:
        gemm("dN2", True, B.NN, B.EPI_NONE, T, H, F1, tf, P["w1"], oth)
    gemm("dA", True, B.NN, B.EPI_NONE, T, A, H, th, P["wo"], ota)
    if post:
        gemm("dX+add", True, B.NN, B.EPI_ADD, T, H, 3 * A, t3a, P["wqkv"], oth, aux_in=res)
    else:
        gemm("dN1", True, B.NN, B.EPI_NONE, T, H, 3 * A, t3a, P["wqkv"], oth)
    wgrad("dW2", H, F, T, th, g)
    wgrad("dW1", F1, H, T, tf, n_in)
    wgrad("dWo", H, A, T, th, attn)
    wgrad("dWqkv", 3 * A, H, T, t3a, n_in)
    n_gemm = len(rows)
    lse_o, delta, dqkv = torch.empty_like(lse), torch.empty_like(lse), torch.empty_like(qkv)
    _, gemm_fwd, att_fwd = layer_flops(cfg, seqlens)
    rows.append(("attention fwd", att_fwd, lambda: B.slapo_attn_fwd(layer.desc, qkv, sld, ota, lse_o), "attn_fwd_bf16_kernel"))
    rows.append(("attention bwd", 2.5 * att_fwd, lambda: B.slapo_attn_bwd(layer.desc, qkv, sld, attn, ta, lse, delta, dqkv),
                 "attn_bwd_*_bf16_kernel"))

    kernels, by_symbol = {}, {}
    for name, flop, fn, symbol in rows:
        ms = timed(fn, reps, stream)
        kernels[name] = {"us": ms * 1e3, "tflops": flop / (ms * 1e-3) / 1e12, "kernel": symbol}
        if name.startswith("dW"):
            s = by_symbol.setdefault(symbol, [0.0, 0.0, 0, []])
            s[0] += flop; s[1] += ms; s[2] += 1; s[3].append(name)
        if verbose:
            print(f"  {name:14s} {ms * 1e3:8.1f} us {flop / ms / 1e9:8.1f} TFLOP/s  {symbol}", file=sys.stderr)
    gemm_ms = sum(kernels[r[0]]["us"] for r in rows[:n_gemm]) * 1e-3
    att_ms = sum(kernels[r[0]]["us"] for r in rows[n_gemm:]) * 1e-3
    gemm_tf = 3.0 * gemm_fwd / (gemm_ms * 1e-3) / 1e12
    att_tf = 3.5 * att_fwd / (att_ms * 1e-3) / 1e12
    joint_tf = (3.0 * gemm_fwd + 3.5 * att_fwd) / ((gemm_ms + att_ms) * 1e-3) / 1e12
    joint = {"gemm_us": gemm_ms * 1e3, "attention_us": att_ms * 1e3,
             "gemm_tflops": gemm_tf, "gemm_frac_of_mfma_peak": gemm_tf / MFMA_BF16_PEAK_TFLOPS,
             "attention_tflops": att_tf, "attention_frac_of_mfma_peak": att_tf / MFMA_BF16_PEAK_TFLOPS,
             "attention_bwd_tflops": kernels["attention bwd"]["tflops"],
             "gemm_attention_tflops": joint_tf, "gemm_attention_frac_of_mfma_peak": joint_tf / MFMA_BF16_PEAK_TFLOPS}

    # Dominant kernel: the weight-gradient (TN) GEMM instance that takes the most time per step (dW2, dW1, dWqkv and,
    # where it is the same instance, dWo), launched through slapo_weight_grad exactly as the layer's backward does.
    symbol, (flop, ms, n, names) = max(by_symbol.items(), key=lambda kv: kv[1][1])
    achieved = flop / (ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"{symbol} (weight gradients {', '.join(names)})",
                "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, symbol)),
                "avg_launch_us": ms * 1e3 / n, "flop_per_launch": flop / n}
    del th, tf, ta, t3a, oth, otf, ota, ot3a, og, res, dqkv

    # HBM-bound fused row kernels. Each launch moves 4 [T,H] tensors (two read, two written); the loop rotates
    # through enough disjoint sets of them that a set has long left the 256 MB last-level cache when its turn
    # comes again.
    eb = 4 if cfg.dtype == W.FP32 else 2
    set_bytes = 4 * T * H * eb
    n_sets = max(4, math.ceil(ROTATE_BYTES / set_bytes))
    sets = [tuple(torch.empty(T, H, device="cuda", dtype=tdt) for _ in range(4)) for _ in range(n_sets)]
    for s in sets:
        s[0].normal_(); s[1].normal_()
    mu = torch.empty(T, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mu)
    gamma, beta, bias = P["ln1_g"], P.get("ln1_b"), P.get("bo")
    it = [0]

    def epi_fwd():   # z = res + drop(r + bias); out = LN(z)
        r, rs, z, o = sets[it[0] % n_sets]
        it[0] += 1
        B.slapo_bdrln_fwd(layer.desc, 0, T, r, bias, rs, gamma, beta, z, o, mu, rstd)

    rounds = max(reps, 2 * n_sets)
    fwd_ms = timed(epi_fwd, rounds, stream, warm=n_sets)
    part = torch.empty(B.slapo_bdrln_bwd_blocks(T) * 3 * H, dtype=torch.float32, device="cuda")

    def epi_bwd():   # dz = LN'(dout; z) ; dr = dz * keep / (1 - p); partial sums of dgamma, dbeta, dbias
        dz, dr, z, dout = sets[it[0] % n_sets]   # (z, dout: what the forward loop left there)
        it[0] += 1
        B.slapo_bdrln_bwd(layer.desc, 0, T, dout, z, mu, rstd, gamma, None, dz, dr, part)

    it[0] = 0
    bwd_ms = timed(epi_bwd, rounds, stream, warm=n_sets)
    del sets
    # context for "achievable" HBM bandwidth: plain device-to-device copies of 256 MiB over rotating buffer pairs
    n_pairs = 4
    pairs = [(torch.empty(256 << 20, dtype=torch.uint8, device="cuda"), torch.empty(256 << 20, dtype=torch.uint8, device="cuda"))
             for _ in range(n_pairs)]

    def copy():
        s, d = pairs[it[0] % n_pairs]
        it[0] += 1
        d.copy_(s)

    copy_ms = timed(copy, 24, stream, warm=n_pairs)
    del pairs
    torch.cuda.empty_cache()

    def hbm(ms, nbytes, note):
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "avg_launch_us": ms * 1e3, "bytes_per_launch": nbytes, "buffers": note}

    note = f"{n_sets} disjoint sets of 4 x [T,H], {n_sets * set_bytes / 2**30:.2f} GiB in rotation"
    hbm_figs = {"epilogue_bdrln_fwd": hbm(fwd_ms, set_bytes, note), "epilogue_bdrln_bwd": hbm(bwd_ms, set_bytes, note),
                "copy_kernel_256MiB": hbm(copy_ms, 2.0 * (256 << 20), f"{n_pairs} disjoint source/destination pairs, 2 GiB in rotation")}
    return kernels, joint, roofline, hbm_figs


def run_config(B, cfg, steps, warmup, stream, checkpoint=0, detail=True, verbose=False):
    """Times the training step of one configuration; with `detail` also its kernels in isolation."""
    params = W.make_params(cfg)
    x, dy, seqlens = W.make_inputs(cfg)
    layer = B.Layer(cfg, params, checkpoint=checkpoint)
    xd, dyd = layer.to_device(x), layer.to_device(dy)
    sld = None if seqlens is None else torch.from_numpy(seqlens).cuda()
    y = torch.empty_like(xd)
    dx = torch.empty_like(xd)

    def step():
        B.slapo_layer_fwd(layer.desc, layer.params, xd, sld, y, layer.saved, layer.scratch)
        B.slapo_layer_bwd(layer.desc, layer.params, xd, sld, dyd, layer.saved, dx, layer.grads, layer.scratch)

    stack = None
    if cfg.n_layers > 1:   # the stack: per-layer weights seeded by the layer index, dy injected at the top
        stack = B.Stack(cfg, [W.make_params(cfg, layer_id=l) for l in range(cfg.n_layers)], checkpoint=checkpoint)

        def step():
            B.slapo_stack_fwd(stack.desc, stack.params, xd, sld, y, stack.acts, stack.saved, stack.scratch)
            B.slapo_stack_bwd(stack.desc, stack.params, xd, sld, dyd, stack.acts, stack.saved, dx, stack.grads,
                              stack.scratch)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    gpu_ms = e0.elapsed_time(e1) / steps
    ms = max(wall_ms, gpu_ms)
    total_flops = layer_flops(cfg, seqlens)[0] * cfg.n_layers
    res = {"workload": cfg.name, "ms_per_step": ms, "gpu_event_ms_per_step": gpu_ms, "wall_ms_per_step": wall_ms,
           "samples_per_s": cfg.batch / (ms * 1e-3), "layer_tflops": total_flops / (ms * 1e-3) / 1e12,
           "layer_frac_of_mfma_peak": total_flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "steps": steps}
    del stack
    torch.cuda.empty_cache()
    if detail and cfg.dtype != W.FP32:
        if checkpoint:   # the isolated-kernel figures read saved activations: take them from a plain layer
            layer = B.Layer(cfg, params)
        kernels, joint, roofline, hbm_figs = kernel_figures(B, cfg, layer, xd, dyd, sld, seqlens, max(20, steps), stream, verbose)
        res.update({"kernels_alone": joint, "kernels": kernels, "roofline": roofline})
        res.update(hbm_figs)
    return res, (params, x, dy, seqlens)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "C6"],
                    help="headline configuration. C5 = the 24-layer stack (one step = 24 layer forwards, then 24 layer "
                         "backwards); C6 = the LLaMA-7B-shaped layer (RMSNorm, rotary, SwiGLU)")
    ap.add_argument("--also", default=None,
                    help="comma-separated configurations whose step figures go under extra.configs "
                         "(default: C3,C4,C5 when the headline is the plain C2 run, else none); 'none' for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--checkpoint", action="store_true",
                    help="activation-checkpointing mode: nothing saved, backward recomputes the forward")
    ap.add_argument("--fp16", action="store_true", help="IEEE half storage instead of bf16 (same kernels)")
    ap.add_argument("--attn-dropout", type=float, default=0.0,
                    help="also drop attention probabilities with this probability (0 = the benchmark configuration)")
    ap.add_argument("--breakdown", action="store_true", help="print the per-kernel table (stderr)")
    ap.add_argument("--layers", type=int, default=0,
                    help="run the configuration as a stack of this many layers (default: the configuration's own count)")
    ap.add_argument("--tp", type=int, default=1,
                    help="time ONE rank's share of the layer sharded N ways along heads and FFN columns "
                         "(heads/N, attention width hidden/N, ffn/N; no collectives are run)")
    ap.add_argument("--eager-baseline", action="store_true",
                    help="also time the same layer as unfused PyTorch library ops with autograd (context, in `extra`)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU sharding is design-only.",
              file=sys.stderr)
        sys.exit(2)

    from paper_2302_08005_amd import binding as B

    cfg = W.CONFIGS[args.config]
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    plain = not (args.attn_dropout or args.fp16 or args.layers or args.tp > 1 or args.checkpoint)
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
    if args.also is None:
        also = ["C3", "C4", "C5"] if (plain and args.config == "C2") else []
    else:
        also = [] if args.also == "none" else [c for c in args.also.split(",") if c]

    head, (params, x, dy, seqlens) = run_config(B, cfg, args.steps, args.warmup, stream, checkpoint=int(args.checkpoint),
                                                verbose=args.breakdown)
    ms = head["ms_per_step"]
    extra = {k: head[k] for k in ("layer_tflops", "layer_frac_of_mfma_peak", "gpu_event_ms_per_step", "wall_ms_per_step")}
    for k in ("kernels_alone", "kernels", "epilogue_bdrln_fwd", "epilogue_bdrln_bwd", "copy_kernel_256MiB"):
        if k in head:
            extra[k] = head[k]
    if args.eager_baseline and cfg.n_layers == 1:
        eager_ms = torch_eager_step_ms(cfg, params, x, dy, seqlens, max(10, args.steps // 2), stream)
        extra["torch_eager_unfused"] = {"ms_per_step": eager_ms, "speedup_of_this_library": eager_ms / ms}
    if also:
        extra["configs"] = {}
        for key in also:
            if args.breakdown:
                print(f"-- {key}", file=sys.stderr)
            res, _ = run_config(B, W.CONFIGS[key], max(10, min(args.steps, 20)), min(args.warmup, 5), stream, verbose=args.breakdown)
            res.pop("kernels", None)   # (the per-kernel table of the other configurations: --config / --breakdown)
            extra["configs"][key] = res

    llama = cfg.arch == W.LLAMA
    out = {"metric": "layer fwd+bwd samples/s", "value": cfg.batch / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": {W.BF16: "bf16", W.FP16: "f16"}.get(cfg.dtype, "f32"),
           "data": "synthetic",
           "config": {"workload": cfg.name, "batch": cfg.batch, "seq": cfg.seq, "hidden": cfg.hidden,
                      "heads": cfg.heads, "ffn": cfg.ffn, "causal": cfg.causal, "dropout_p": cfg.dropout_p,
                      "attn_dropout_p": cfg.attn_dropout_p, "pre_ln": cfg.pre_ln, "layers": cfg.n_layers, "checkpoint": int(args.checkpoint),
                      "family": "llama" if llama else "classic", "tp_share": args.tp,
                      "parallelism": "single-gpu"},
           "roofline": head.get("roofline"), "extra": extra}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, params, x, dy, seqlens)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
