#!/usr/bin/env python3
"""StreamBP backward benchmark: one 7B-shaped decoder layer + LM head at 32k tokens (the headline workload; the
other workloads of the paper's shape list can be timed with --workload).

A step = one pass of the whole hot path over one synthetic sequence:
LM-head + cross-entropy StreamBP (chunk 2048 rows of logits at a time) followed
by the layer-wise StreamBP of one decoder layer (K/V pre-pass, then per chunk:
reforward, MLP / attention backward, dW accumulation), with all inputs already
resident in HBM.  Prints ONE JSON line (see README for the fields).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b|llama_layer|lmhead|grpo|stack] [--seq-len T]
                    [--chunk C] [--batch B] [--prompt-frac P] [--layers L] [--grad-dtype f32|bf16] [--no-cpu-baseline]
                    [--no-profile]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # 256 CU x 4096 flop/clk/CU x 2.4 GHz (dense bf16 MFMA); vendor figure ~2.5 PF
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel of the default workload.  Hardware counters cannot be read inside
# the timed process: the figure is the one two rocprofv3 --pmc runs of this script measured (FETCH_SIZE, WRITE_SIZE, scaled
# by a 1 GiB copy-like kernel) and is reported together with the file under profiles/ that holds those runs; for any
# other kernel or shape the field is null.
MEASURED_TRAFFIC = {      # kernel symbol -> (bytes per launch, file under profiles/)
    "gemm_mfma_k<false, false, 3>": (1.374e9, "profiles/bench_7b_layer_lmhead_32k_hbm_traffic.txt"),
}


def algorithmic_flops(cfg, T, active_rows, batch=1, has_layer=True, has_head=True, n_layers=1, lora_rank=0, window=0):
    """Work the method must do (Sec. 3.2): 6*P per token for the linear maps (reforward, dX, dW), 14*dh per
    visible causal (query, key) pair per query head (4 forward + 10 backward), 6*d*V per row of the head.
    T = tokens per sequence, batch sequences (no attention across sequences), active_rows over the whole batch."""
    d = cfg["hidden"]
    linear = attn = head_all = head_active = 0.0
    if has_layer:
        Hq, Hkv, dh, F = (cfg[k] for k in ("n_q_heads", "n_kv_heads", "head_dim", "mlp_width"))
        p_lin = d * Hq * dh + 2 * d * Hkv * dh + Hq * dh * d + 3 * d * F
        linear = 6.0 * p_lin * T * batch * n_layers
        if lora_rank:   # adapter mode: reforward and dX at the effective matrices, no dW; four rank-r products per adapted matrix
            dims = 2 * (d + Hq * dh) + 2 * (d + Hkv * dh) + 3 * (d + F)        # sum of (in + out) over the seven matrices
            linear = (4.0 * p_lin + 8.0 * lora_rank * dims) * T * batch * n_layers
        pairs = T * (T + 1) / 2.0
        if window and window < T:                                              # visible (query, key) pairs under a sliding window
            pairs = window * (window + 1) / 2.0 + (T - window) * float(window)
        attn = 14.0 * dh * Hq * pairs * batch * n_layers
    if has_head:
        V = cfg["vocab"]
        head_all = 6.0 * d * V * T * batch
        head_active = 6.0 * d * V * active_rows
    # Rows whose target is ignored (prompt positions) need no head work at all (their dz is zero) and the
    # library skips them, so only the active rows are credited; the all-rows figure is kept for reference.
    return dict(linear=linear, attention=attn, head_all_rows=head_all, head_active_rows=head_active,
                total=linear + attn + head_active, total_all_rows=linear + attn + head_all,
                # per GEMM family (forward NT, input-gradient NN, weight-gradient TN): a third of the linear work each
                gemm_family=(linear + head_active) / 3.0)


def cpu_baseline(cfg, seconds_hint=20.0):
    """The fp64 oracle as it stands, timed on this machine's host cores on a bounded sample of the same
    workload: one 7B-shaped layer forward+backward at T_s tokens and the LM head on R_s rows."""
    import numpy as np
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    from oracle import head as o_head
    from oracle import layer as o_layer
    from paper_2506_03077_amd import synth
    T_s, R_s = 4096, 1536
    lc = dict(cfg, dtype="bf16")
    inp = synth.layer_inputs(lc, seed=0, seq_len=T_s, batch=1)
    ocfg = dict(n_q_heads=cfg["n_q_heads"], n_kv_heads=cfg["n_kv_heads"], head_dim=cfg["head_dim"])
    t0 = time.perf_counter()
    o_layer.layer_forward_backward(inp["x"], inp["w"], ocfg, inp["dy"])
    t_layer = time.perf_counter() - t0
    hin = synth.head_inputs(lc, seed=0, seq_len=R_s, batch=1, prompt_frac=0.0)
    t0 = time.perf_counter()
    o_head.sft(hin["h"], hin["w"], hin["targets"], 1.0 / R_s)
    t_head = time.perf_counter() - t0
    per_token = t_layer / T_s + t_head / R_s
    return dict(value=1.0 / per_token, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=(f"fp64 numpy oracle, full-sequence backprop: one layer fwd+bwd at T={T_s} ({t_layer:.1f} s) + "
                        f"LM head on {R_s} rows ({t_head:.1f} s), 7B-shaped widths; per-token times added "
                        f"(attention cost at T={T_s}, not 32k)"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", choices=("7b", "llama_layer", "lmhead", "grpo", "stack"), default="7b",
                    help="7b (default, the workload the metric is quoted on): 7B-shaped layer + LM head, 32k tokens, SFT on all "
                         "positions; llama_layer: one Llama-style layer, 8k tokens; lmhead: LM head + cross-entropy only, 32k rows, "
                         "first 25%% ignored; grpo: 7B-shaped layer + LM head, 8 sequences x 16k tokens, GRPO objective, response = "
                         "last 75%%; stack: the whole 7B-shaped stack (28 layers + head) from per-layer checkpoints")
    ap.add_argument("--prompt-frac", type=float, default=None,
                    help="fraction of every sequence, from its start, whose targets are ignored (default: 0 for 7b / stack - "
                         "SFT on all positions - and 0.25 for lmhead / grpo, as their workloads say)")
    ap.add_argument("--layers", type=int, default=None, help="stack workload: number of layers (default 28)")
    ap.add_argument("--lora-rank", type=int, default=0,
                    help="7b / llama_layer / grpo: run the layer in adapter mode (rank-R adapters on all seven matrices, adapter "
                         "gradients only; the paper's setting for its largest model is R = 32)")
    ap.add_argument("--window", type=int, default=0, help="sliding-window attention in the layer (0 = plain causal)")
    ap.add_argument("--grad-dtype", choices=("f32", "bf16"), default="f32",
                    help="element type of the weight-gradient accumulators (default fp32; bf16 is the paper's own training "
                         "setting, App. D (experiment setup), and halves the read-modify-write traffic on dW)")
    ap.add_argument("--dw-group-rows", type=int, default=0,
                    help="rows of chunk operands kept alive per pass over the weight gradients (0 = the library's defaults: 8192 for the layer, 16384 for the head)")
    ap.add_argument("--batch", type=int, default=None, help="sequences per call (default: the workload's own)")
    ap.add_argument("--seq-len", type=int, default=None)
    ap.add_argument("--chunk", type=int, default=None)
    ap.add_argument("--head-chunk", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--fusions", type=int, default=None,
                    help="A/B: bit mask of the optional fusions of the layer path (see include/streambp_debug.h); default: the library's")
    ap.add_argument("--no-masked-run", action="store_true",
                    help="skip the second timing of the default workload with the first 25%% of the positions ignored")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the pure-MFMA rate probe that runs after the timed steps (config.mfma_only_sustained_tflops)")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run one plain elementwise kernel that reads 1 GiB and writes 1 GiB (reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc runs (goes into roofline.traffic)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_03077_amd import binding as sb
    from paper_2506_03077_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sb.lib()   # fails loudly if the HIP library is missing
    if args.fusions is not None:
        sb.debug_set_fusions(args.fusions)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = args.workload
    stack = wl == "stack"
    cfg = dict(synth.CONFIGS["7b" if stack else wl])
    has_layer, has_head = wl != "lmhead", wl != "llama_layer"
    grpo = wl == "grpo"
    B = args.batch or cfg["batch"]
    T = args.seq_len or cfg["seq_len"]
    c = args.chunk or cfg["chunk"]
    hc_rows = args.head_chunk or c
    L = (args.layers or cfg["n_layers"]) if stack else 1
    prompt_frac = args.prompt_frac if args.prompt_frac is not None else (0.25 if wl in ("lmhead", "grpo") else 0.0)
    gdt = sb.SBP_BF16 if args.grad_dtype == "bf16" else sb.SBP_F32
    default_shape = (wl == "7b" and T == cfg["seq_len"] and c == cfg["chunk"] and hc_rows == c and B == cfg["batch"]
                     and not args.lora_rank and not args.window and prompt_frac == 0.0 and gdt == sb.SBP_F32 and args.dw_group_rows == 0)   # what the profiles cover
    d = cfg["hidden"]
    bf = torch.bfloat16

    # ---- synthetic inputs, generated on the device (seeded): weights N(0, 0.02), hidden states N(0, 1),
    # gains 1 + N(0, 0.02), upstream gradients N(0, 1e-3), target ids uniform in [0, V); the first prompt_frac of the
    # positions of every sequence ignored (prompt); GRPO: advantages N(0, 1) per sequence, reference log-probs
    # N(-2, 0.5), on-policy (no old log-probs).
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def normal(shape, std, mean=0.0):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std + mean).to(bf)

    n_prompt = int(round(prompt_frac * T))
    n_act = B * (T - n_prompt)
    ws_bytes = {}

    def layer_weights():
        Hq, Hkv, dh, F = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["mlp_width"]
        return dict(wq=normal((Hq * dh, d), 0.02), wk=normal((Hkv * dh, d), 0.02), wv=normal((Hkv * dh, d), 0.02),
                    wo=normal((d, Hq * dh), 0.02), wgate=normal((F, d), 0.02), wup=normal((F, d), 0.02),
                    wdown=normal((d, F), 0.02), g1=normal((d,), 0.02, 1.0), g2=normal((d,), 0.02, 1.0))

    if has_layer:
        Hq, Hkv, dh, F = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["mlp_width"]
        lcfg = sb.layer_cfg(sb.SBP_BF16, B, T, c, d, Hq, Hkv, dh, F, grad_dtype=gdt, dw_group_rows=args.dw_group_rows,
                            window=args.window)
        assert sb.streambp_layer_fast_path(lcfg) == 1, sb.streambp_last_error()
        ws_bytes["layer_workspace"] = sb.streambp_layer_workspace_bytes(lcfg)
    if has_head:
        V = cfg["vocab"]
        targets = torch.randint(0, V, (B, T), generator=gen, device=dev, dtype=torch.int32)
        targets[:, :n_prompt] = -1
        adv = ref_logp = None
        if grpo:
            adv = torch.randn((B,), generator=gen, device=dev, dtype=torch.float32)
            ref_logp = torch.randn((B, T), generator=gen, device=dev, dtype=torch.float32) * 0.5 - 2.0
            hcfg = sb.head_cfg(sb.SBP_BF16, B, T, hc_rows, d, V, sb.SBP_OBJ_GRPO, grad_dtype=gdt, dw_group_rows=args.dw_group_rows)
        else:
            hcfg = sb.head_cfg(sb.SBP_BF16, B, T, hc_rows, d, V, sb.SBP_OBJ_SFT, 1.0 / n_act, grad_dtype=gdt, dw_group_rows=args.dw_group_rows)
        assert sb.streambp_lmhead_fast_path(hcfg) == 1, sb.streambp_last_error()
        ws_bytes["head_workspace"] = sb.streambp_lmhead_workspace_bytes(hcfg)
        ws_bytes["full_sequence_logits_fp32_would_be"] = B * T * V * 4
        w_head = normal((V, d), 0.02)
        dw_head = torch.zeros((V, d), dtype=torch.bfloat16 if gdt == sb.SBP_BF16 else torch.float32, device=dev)
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        n_active = torch.zeros(1, dtype=torch.int64, device=dev)

    if stack:
        # Whole stack: the chunked forward fills one checkpoint per layer (untimed here: the metric is the backward),
        # then the timed step is streambp_stack_backward = final norm, LM head, L x layer StreamBP, embedding scatter-add.
        layers = [layer_weights() for _ in range(L)]
        g_final = normal((d,), 0.02, 1.0)
        emb = normal((V, d), 0.02)
        ids = torch.randint(0, V, (B, T), generator=gen, device=dev, dtype=torch.int32)
        scfg = sb.stack_cfg(lcfg, L, V, hc_rows, sb.SBP_OBJ_SFT, 1.0 / n_act)
        ws_stack = torch.empty(sb.streambp_stack_workspace_bytes(scfg), dtype=torch.uint8, device=dev)
        ws_bytes["stack_workspace"] = ws_stack.numel()
        ckpt = [torch.empty((B, T, d), dtype=bf, device=dev) for _ in range(L + 1)]
        ws_bytes["checkpoints"] = sum(t.numel() * 2 for t in ckpt)
        t0 = time.perf_counter()
        sb.streambp_stack_forward(scfg, layers, ckpt, emb=emb, ids=ids, workspace=ws_stack)
        torch.cuda.synchronize()
        forward_s = time.perf_counter() - t0
        grads = dict(dlayers=[sb.new_layer_grads(w, gdt) for w in layers], dg_final=torch.zeros(d, dtype=torch.float32, device=dev),
                     dw_head=dw_head, demb=torch.zeros((V, d), dtype=torch.float32, device=dev),
                     dx0=torch.empty((B, T, d), dtype=bf, device=dev), loss=loss, n_active=n_active)

        def step():
            sb.streambp_stack_backward(scfg, layers, g_final, w_head, ckpt, targets, ids=ids, workspace=ws_stack, **grads)
        dx = grads["dx0"]
    else:
        if has_layer:
            w = layer_weights()
            x = normal((B, T, d), 1.0)          # layer input (the checkpoint)
            if args.lora_rank:
                r = args.lora_rank
                adapters = {n: (normal((r, w[n].shape[1]), 0.02), normal((w[n].shape[0], r), 0.02)) for n in sb.MATRIX_NAMES}
                ws_bytes["layer_workspace"] = sb.streambp_layer_lora_workspace_bytes(lcfg, adapters, r, 2.0)
                da = {n: torch.zeros(ab[0].shape, dtype=torch.float32, device=dev) for n, ab in adapters.items()}
                db = {n: torch.zeros(ab[1].shape, dtype=torch.float32, device=dev) for n, ab in adapters.items()}
            ws_layer = torch.empty(ws_bytes["layer_workspace"], dtype=torch.uint8, device=dev)
            dw = sb.new_layer_grads(w, gdt)
            dx = torch.empty_like(x)
        if has_head:
            h = normal((B, T, d), 1.0)          # hidden states entering the head
            ws_head = torch.empty(ws_bytes["head_workspace"], dtype=torch.uint8, device=dev)
            dh_out = torch.empty_like(h)
        else:
            dh_out = normal((B, T, d), 1e-3)    # upstream gradient of the layer

        def step():
            if has_head:
                sb.streambp_lmhead_ce_backward(hcfg, w_head, h, targets, ref_logp=ref_logp, advantages=adv, dh=dh_out, dw=dw_head,
                                               loss=loss, n_active=n_active, workspace=ws_head)
            if has_layer:
                # the head's dH is the upstream gradient of the layer (the final norm is left out of the timed step)
                if args.lora_rank:
                    sb.streambp_layer_lora_backward(lcfg, w, adapters, args.lora_rank, 2.0, x, dh_out, dx=dx, da=da, db=db, workspace=ws_layer)
                else:
                    sb.streambp_layer_backward(lcfg, w, x, dh_out, dx=dx, dw=dw, workspace=ws_layer)

    if args.pmc_calibrate:   # 2^28 fp32 elements: the add kernel fetches 1 GiB and writes 1 GiB
        ca = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        cb = torch.empty_like(ca)
        torch.add(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb

    def timed(n_warm, n_steps):
        for _ in range(n_warm):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / max(n_steps, 1)

    generic_before = sb.streambp_generic_launches()
    dt = timed(args.warmup, args.steps)
    assert sb.streambp_generic_launches() == generic_before, "a launch left the MFMA kernels"

    if has_head:
        assert int(n_active.item()) == n_act
        assert bool(torch.isfinite(loss).all())
        if not stack:
            assert bool(torch.isfinite(dh_out.float()).all())
    if has_layer:
        assert bool(torch.isfinite(dx.float()).all())

    fl = algorithmic_flops(cfg, T, n_act, B, has_layer, has_head, L, args.lora_rank, args.window)
    names = {"7b": "7B-shaped decoder layer (d=3584, 28q/4kv x128, F=18944) + LM head (V=152064)",
             "llama_layer": "Llama-style decoder layer (d=4096, 32q/8kv x128, F=14336), upstream gradient N(0,1e-3)",
             "lmhead": "LM head + cross-entropy (d=3584, V=152064)",
             "grpo": "7B-shaped decoder layer + LM head (V=152064), GRPO objective (on-policy, reference log-probs)",
             "stack": f"7B-shaped stack: {L} decoder layers (d=3584, 28q/4kv x128, F=18944) from per-layer checkpoints + final norm "
                      f"+ LM head (V=152064) + embedding gradient"}
    loss_on = ("loss on all positions" if n_prompt == 0 else
               f"loss on the last {100 * (T - n_prompt) / T:.0f}% of the positions of every sequence (the rest ignored)")
    out = {
        "metric": "backward tokens/s per layer+LM head at 32k seq" if not stack else "backward tokens/s, whole stack at 32k seq",
        "value": B * T / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{names[wl]}, T={T}, chunk={c}, head chunk={hc_rows}, batch {B}, {loss_on}, "
                               f"{args.grad_dtype} weight-gradient accumulators"
                               + (f", layer in adapter mode (rank {args.lora_rank} on all seven matrices, adapter gradients only)" if args.lora_rank else "")
                               + (f", sliding window {args.window}" if args.window else "")
                               + (f", weight gradients added once per {args.dw_group_rows} rows" if args.dw_group_rows else ""),
                   "algorithmic_tflop_per_step": fl["total"] / 1e12,
                   "achieved_tflops": fl["total"] / dt / 1e12,
                   "frac_of_bf16_mfma_peak": fl["total"] / dt / 1e12 / PEAK_BF16_TFLOPS,
                   "peak_activation_bytes": ws_bytes,
                   "torch_max_memory_allocated": int(torch.cuda.max_memory_allocated())},
    }
    if n_prompt:
        out["config"]["algorithmic_tflop_per_step_if_ignored_rows_were_counted"] = fl["total_all_rows"] / 1e12
    if stack:
        out["config"]["forward_with_checkpoints_s"] = forward_s

    # ---- roofline of the dominant kernel (largest total time), durations from HIP events recorded on the
    # launch stream around every launch during one more pass over the same workload.
    if not args.no_profile:
        sb.debug_profile_begin(20000 * max(1, L // 4))
        step()
        torch.cuda.synchronize()
        prof = sb.debug_profile_end()
        # Flops per kernel: 2MNK summed over its launches.  For the LM-head GEMMs the row count of a chunk lives
        # on the device (ignored rows are compacted away), so the library reports their work from the host-side
        # upper bound separately; the real row total is n_active of B*T rows, hence the factor below.
        active_frac = n_act / float(B * T)
        per_kernel = {}
        for kname, v in prof.items():
            if not v["count"]:
                continue
            fl_k = v["flops"] + v["flops_bounded"] * active_frac
            per_kernel[kname] = dict(launches=v["count"], ms=v["ms"], avg_launch_ms=v["ms"] / v["count"],
                                     tflops=fl_k / v["ms"] / 1e9, tflop=fl_k / 1e12)
        dom = max(per_kernel, key=lambda kname: per_kernel[kname]["ms"])
        pk = per_kernel[dom]
        traffic = MEASURED_TRAFFIC.get(dom) if default_shape else None
        if args.traffic_bytes is not None:
            traffic = (args.traffic_bytes, "command line (--traffic-bytes)")
        out["roofline"] = {"bound": "mfma", "kernel": dom, "launches_per_step": pk["launches"],
                           "avg_launch_ms": pk["avg_launch_ms"], "avg_launch_tflop": pk["tflop"] / pk["launches"],
                           "achieved": pk["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": pk["tflops"] / PEAK_BF16_TFLOPS,
                           "traffic": traffic[0] if traffic else None,
                           "traffic_source": traffic[1] if traffic else None}
        out["config"]["per_kernel"] = per_kernel

    # ---- second figure for the default workload: the same step with the first quarter of the positions ignored (the
    # prompt mask of the LM-head workload of the shape list); the library compacts those rows away.
    if default_shape and not args.no_masked_run:
        n_prompt2 = T // 4
        targets[:, :n_prompt2] = -1
        n_act2 = B * (T - n_prompt2)
        hcfg.loss_scale = 1.0 / n_act2
        dt2 = timed(1, max(1, min(args.steps, 3)))
        fl2 = algorithmic_flops(cfg, T, n_act2, B, has_layer, has_head, L)
        out["config"]["same_step_with_first_25pct_of_positions_ignored"] = dict(
            ms_per_step=dt2 * 1e3, tokens_per_s=B * T / dt2, algorithmic_tflop_per_step=fl2["total"] / 1e12,
            achieved_tflops=fl2["total"] / dt2 / 1e12, frac_of_bf16_mfma_peak=fl2["total"] / dt2 / 1e12 / PEAK_BF16_TFLOPS)
    # ---- context for the roofline fractions: what the matrix pipe sustains with NO global memory traffic at all (eight
    # independent MFMAs per wave and round, two waves per SIMD).  The chip is power-managed, so the rate depends on the operand
    # values: all-zero fragments reach the nominal peak, random ones (what every GEMM of the path multiplies) do not - and
    # less again when the fragments come from LDS the way the kernels' main loops fetch them (6 reads of 1 KB per 8 products
    # in the GEMMs, 8 in the attention backward).
    if not args.no_profile and not args.no_mfma_probe:
        zeros = torch.zeros(32768, dtype=torch.bfloat16, device=dev)
        rnd = normal((32768,), 1.0)
        out["config"]["mfma_only_sustained_tflops"] = {
            "zero_operands": sb.debug_mfma_rate(zeros), "random_operands": sb.debug_mfma_rate(rnd),
            "random_operands_6_lds_fragment_reads_per_8_mfma": sb.debug_mfma_rate(rnd, lds_reads=6),
            "random_operands_8_lds_fragment_reads_per_8_mfma": sb.debug_mfma_rate(rnd, lds_reads=8),
            "how": "streambp_debug_mfma_rate: 12 launches of 512 workgroups x 8 waves x 10000 rounds of 8 v_mfma_f32_32x32x16_bf16, no global loads"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(dict(synth.CONFIGS["7b"]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
