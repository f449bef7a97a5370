#!/usr/bin/env python3
"""Benchmark of the padding-free MoE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dsmoe16b]

A step is one pass of the whole hot path - gate projection, routing, ERI construction, dispatch, expert MLP
(routed + shared), combine, and the complete backward (combine bwd, expert MLP dgrad + wgrad, dispatch bwd,
routing bwd, gate projection bwd) - over one batch of synthetic tokens that is already resident in HBM.
Prints ONE JSON line: tokens/s for forward+backward, the roofline figures of the dominant kernel measured live
with HIP events on the launch stream, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0               # MI355X HBM3E, published
PEAK_FP32_TFLOPS = 157.3            # MI355X float32 vector / matrix, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="dsmoe16b",
                    help="dsmoe16b (default, the config the metric is quoted on), dsmoe16b_skew, large, longseq[-T<N>], ...")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--max-token-count", type=int, default=None,
                    help="run the layer with the token-dropping PFT construction at this per-expert capacity "
                         "(default: dropless, the configuration the metric is quoted on)")
    ap.add_argument("--materialise-dy", action="store_true",
                    help="unfused backward of combine: dY [B,d] is written and read back (for comparisons)")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as one replay of a captured HIP graph instead of two dozen launches")
    ap.add_argument("--rbd-experts-per-node", type=int, default=0,
                    help="also time stage 0 of the redundancy-bypassing dispatch on this layer's routing with that "
                         "many experts per destination node (reported beside the step, not part of it)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run the library's plain copy kernel once over 1 GiB (a kernel of known traffic, "
                         "for scaling hardware byte counters under rocprofv3 --pmc)")
    return ap.parse_args()


def get_cfg(name):
    import xmoe_inputs as xi
    if name.startswith("longseq-T"):
        return xi.CONFIGS["longseq"].with_T(int(name[len("longseq-T"):]))
    return xi.CONFIGS[name]


def small_kernel_work(cfg):
    """Algorithmic bytes of the index kernels and float32 flops of the gate projection kernels (both expert kinds)."""
    T, d, E, k, B = cfg.T, cfg.d, cfg.E, cfg.k, cfg.B
    chunks = (B + 1023) // 1024
    bytes_ = {
        "eri_hist_kernel": B * 4 + chunks * E * 4,                    # expert ids read, chunk histograms written
        "eri_scan_kernel": 2 * chunks * E * 4 + (2 * E + 1) * 4,      # histograms -> chunk bases, counts, offsets
        "eri_scatter_kernel": B * 8 + chunks * E * 4 + B * 16,        # (expert, weight) read; 4 arrays of B written
    }
    f32_flops = {"gate_logits_kernel": 2 * T * d * E, "gate_bwd_dw_kernel": 2 * T * d * E,
                 "gate_bwd_dx_kernel": 2 * T * d * E}
    # bf16 workloads with d % 64 == 0 and E % 64 == 0: the two backward products run on the bf16 matrix instruction
    # (dlogits as two bf16 terms, i.e. twice these flops are executed)
    bf16_mfma = {}
    if cfg.dtype == "bf16" and d % 64 == 0 and E % 64 == 0:
        bf16_mfma = {k_: f32_flops.pop(k_) for k_ in ("gate_bwd_dw_kernel", "gate_bwd_dx_kernel")}
    return bytes_, f32_flops, bf16_mfma


def kernel_work(cfg, materialise_dy=False):
    """Algorithmic work of one step per kernel: flops for the GEMM kernels, bytes for the row movers.
    The expert MLP runs on R = B + E_s*T rows (the shared experts' segments are copies of x).
    materialise_dy: the unfused backward of combine (dY written by combine_bwd, dOut copied to the shared rows)."""
    dy_rows = 1 if materialise_dy else 0
    s = 4 if cfg.dtype == "f32" else 2
    T, d, E, k, f, B = cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, cfg.B
    Ts = cfg.E_s * T
    rf = (B + Ts) * f
    if cfg.expert == "mlp2":
        # the paper's two-matrix expert: four row GEMMs of 2*R*d*f flops and two weight gradients
        R, W = B, E * d * f * s
        flops = {"up": 2 * d * rf, "down": 2 * d * rf, "dact": 2 * d * rf, "dx": 2 * d * rf, "wgrad": 4 * d * rf,
                 "bwd_rest": 6 * d * rf}       # dXd, dW2 and dW1 as one launch
        bytes_ = {
            "combine_kernel": (B + T) * d * s + (B + 2 * T) * d * s,
            "combine_bwd_kernel": (T + (1 + dy_rows) * B) * d * s,
            "row_grad_reduce_kernel": ((f + 255) // 256 * 4 + 1) * B * 4,
            "combine_bwd_weights_kernel": B * 12,
            "route_kernel": T * E * 4 + T * k * 8,
            "route_bwd_kernel": 2 * T * E * 4 + T * k * 8,
        }
        gemm_bytes = {"up": R * d * s + W + 2 * R * f * s, "down": R * f * s + W + R * d * s,
                      "dact": R * d * s + W + 3 * R * f * s, "dx": R * f * s + W + R * d * s,
                      "wgrad": 2 * (R * f * s + R * d * s + W)}
        gemm_bytes["bwd_rest"] = gemm_bytes["dx"] + gemm_bytes["wgrad"]
        bytes_.update({"gemm:" + k_: v for k_, v in gemm_bytes.items()})
        return flops, bytes_
    flops = {"gateup": 4 * d * rf, "down": 2 * d * rf, "dact": 2 * d * rf, "dx": 4 * d * rf, "wgrad": 6 * d * rf,
             "wgrad_wd": 2 * d * rf, "wgrad_wg_wu": 4 * d * rf,
             "bwd_rest": 10 * d * rf}          # dXd, dWd and dWg | dWu as one launch
    bytes_ = {
        # only use left in the layer: the unfused backward (E_s > 0), dout copied to the shared experts' dY rows
        "dispatch_kernel": (T + Ts) * d * s if (Ts and materialise_dy) else 0,
        "combine_kernel": (B + Ts + T) * d * s                                # forward combine
                          + (B + Ts + 2 * T) * d * s,                         # + dispatch backward (same kernel)
        # only with --materialise-dy: the fused backward takes the combine weights' gradient from the dAct GEMM
        "combine_bwd_kernel": (T + (1 + dy_rows) * B) * d * s,
        "row_grad_reduce_kernel": ((f + 255) // 256 * 4 + 1) * (B + Ts) * 4,
        "combine_bwd_weights_kernel": B * 12,
        "route_kernel": T * E * 4 + T * k * 8,
        "route_bwd_kernel": 2 * T * E * 4 + T * k * 8,
    }
    # algorithmic bytes of the GEMM kernels: every operand read once, every result written once
    R, W = B + Ts, (E + cfg.E_s) * d * f * s
    gemm_bytes = {"gateup": R * d * s + 2 * W + 3 * R * f * s, "down": R * f * s + W + R * d * s,
                  "dact": R * d * s + W + 5 * R * f * s, "dx": 2 * R * f * s + 2 * W + R * d * s,
                  "wgrad_wd": R * f * s + R * d * s + W, "wgrad_wg_wu": R * d * s + 2 * R * f * s + 2 * W}
    gemm_bytes["wgrad"] = gemm_bytes["wgrad_wd"] + gemm_bytes["wgrad_wg_wu"]
    gemm_bytes["bwd_rest"] = gemm_bytes["dx"] + gemm_bytes["wgrad"]
    bytes_.update({"gemm:" + k_: v for k_, v in gemm_bytes.items()})
    return flops, bytes_


# profiler kernel name -> entry of kernel_work()'s flop table
GEMM_WORK = {
    "ffn_gateup_dma_kernel": "gateup", "ffn_rowgemm_dma_kernel<false>": "down",
    "ffn_rowgemm_dma_kernel<true>": "dact", "ffn_dx_dma_kernel": "dx",
    "ffn_wgrad_dma_kernel<false>": "wgrad_wd", "ffn_wgrad_dma_kernel<true>": "wgrad_wg_wu",
    "ffn_bwd_rest_dma_kernel": "bwd_rest",
}
for _fam in ("mfma", "simt"):
    for _k in ("gateup", "down", "dact", "dx", "wgrad"):
        GEMM_WORK[f"ffn_{_k}_{_fam}_kernel"] = _k
# the two-matrix expert shares the down, dX and weight-gradient kernels (two launches of the latter per step)
GEMM_WORK_MLP2 = {
    "mlp2_up_dma_kernel": "up", "ffn_rowgemm_dma_kernel<false>": "down", "mlp2_dact_dma_kernel": "dact",
    "ffn_dx_dma_kernel": "dx", "ffn_wgrad_dma_kernel<false>": "wgrad", "ffn_bwd_rest_dma_kernel": "bwd_rest",
    "mlp2_up_simt_kernel": "up", "ffn_down_simt_kernel": "down", "mlp2_dact_simt_kernel": "dact",
    "ffn_dx_simt_kernel": "dx", "ffn_wgrad_simt_kernel": "wgrad",
}

def load_measured_traffic(workload):
    """HBM bytes per launch of every kernel as read from the hardware counters (rocprofv3 --pmc FETCH_SIZE, then
    WRITE_SIZE, each scaled by what the same counter shows for xmoe_prof_copy's known traffic): parsed from the
    committed summary profiles/layer_<workload>_dma_family_hbm_traffic.txt, whose header states the commands.
    Keys are the event profiler's kernel names (name + first template argument).  {} if no summary exists."""
    import re
    path = os.path.join(ROOT, "profiles", f"layer_{workload}_dma_family_hbm_traffic.txt")
    out = {}
    if not os.path.exists(path):
        return out
    for ln in open(path):
        m = re.match(r"^([a-z0-9_]+)(?:<([^>]*)>)?\s+(\d+)\s+(\d+)\s+(\d+)\s+(\d+)\s*$", ln)
        if not m:
            continue
        name, targs = m.group(1), (m.group(2) or "").split(",")[0].strip()
        if targs in ("true", "false"):
            out[f"{name}<{targs}>"] = int(m.group(6))
        out.setdefault(name, int(m.group(6)))
    return out


def parity_against(ref, got):
    """(max over rows of ||got_r - ref_r|| / ||ref_r||, max over elements of |got - ref| / max(|ref|, row RMS)): the two
    figures of the whole-layer bf16 criterion (tests/gpu_util.py assert_close_chain)."""
    import numpy as np
    n = np.sqrt((ref * ref).sum(axis=-1))
    e = np.sqrt(((got - ref) ** 2).sum(axis=-1))
    row = float((e / np.where(n == 0.0, 1.0, n)).max())
    rms = np.sqrt((ref * ref).mean(axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), rms)
    el = float((np.abs(got - ref) / np.where(den == 0.0, 1.0, den)).max())
    return round(row, 5), round(el, 5)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2508_13337_amd as xm
    import xmoe_inputs as xi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = get_cfg(args.workload)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(tdt).cuda()

    t_gen = time.time()
    x_np, dout_np = xi.make_x(cfg), xi.make_dout(cfg)
    wr_np, bias_np = xi.make_w_router(cfg), xi.make_gate_bias(cfg)
    w = {"w_router": dev(wr_np), "bias": None if bias_np is None else torch.from_numpy(bias_np).cuda()}
    mlp2 = cfg.expert == "mlp2"
    wkeys = ("w1", "w2") if mlp2 else ("wg", "wu", "wd")
    for key in wkeys:
        # expert by expert, so that the large workloads never hold a second host copy of a whole tensor
        Ea = cfg.E + cfg.E_s   # the shared experts' weights follow the routed ones
        shape = (Ea, cfg.d, cfg.f) if key not in ("wd", "w2") else (Ea, cfg.f, cfg.d)
        w[key] = torch.empty(shape, dtype=tdt, device="cuda")
        for e, a in xi.iter_expert_weights(cfg, key):
            w[key][e].copy_(dev(a))
        if cfg.E_s:
            w[key][cfg.E:].copy_(dev(xi.make_shared_weights(cfg, key)))
    grads = {"dw_router": torch.empty_like(w["w_router"])}
    for key in wkeys:
        grads["d" + key] = torch.empty_like(w[key])
    x, dout = dev(x_np), dev(dout_np)
    if mlp2:
        assert cfg.E_s == 0 and args.max_token_count is None
        layer = xm.XMoE2Layer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, tdt, act=cfg.act,
                              fuse_combine_bwd=not args.materialise_dy)
    else:
        layer = xm.XMoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, tdt, E_s=cfg.E_s,
                             max_token_count=args.max_token_count, fuse_combine_bwd=not args.materialise_dy)
    t_gen = time.time() - t_gen

    def eager_step():
        layer.forward(x, w)
        layer.backward(x, w, dout, grads)

    step = eager_step
    if args.graph:
        graph = xm.capture_step(layer, x, w, dout, grads)
        step = graph.replay

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        xm.xmoe_prof_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    # what a plain copy kernel reaches on this GPU (read + written bytes per second): the practical ceiling that the
    # HBM-bound kernels are to be read against, next to the published 8 TB/s that the roofline fractions use
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(2):
        xm.xmoe_prof_copy(src, dst)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        xm.xmoe_prof_copy(src, dst)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * (1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst
    # and what the vendor library's dense bf16 GEMM reaches on this machine for one [65536,2048] x [2048,2816] product
    # (the gate/up GEMM of config 2 without raggedness, gather or epilogue): the attainable matrix-core rate under the
    # clock the chip really holds.  Measurement only; nothing of the hot path runs through it.
    ma = torch.randn(65536, 2048, device="cuda").to(torch.bfloat16)
    mb = torch.randn(2048, 2816, device="cuda").to(torch.bfloat16)
    for _ in range(3):
        torch.matmul(ma, mb)
    ev0.record()
    for _ in range(10):
        torch.matmul(ma, mb)
    ev1.record()
    torch.cuda.synchronize()
    dense_tflops = 10 * 2 * 65536 * 2048 * 2816 / (ev0.elapsed_time(ev1) * 1e-3) / 1e12
    del ma, mb

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)

    # forward-only timing (reported, not the metric)
    torch.cuda.synchronize()
    tf0 = time.perf_counter()
    for _ in range(args.steps):
        layer.forward(x, w)
    torch.cuda.synchronize()
    fwd_ms = (time.perf_counter() - tf0) * 1e3 / args.steps

    # per-kernel durations: the same steps again with every kernel launch bracketed by HIP events on the
    # launch stream (kept out of the throughput measurement above)
    xm.xmoe_prof_reset()
    xm.xmoe_prof_enable(True)
    for _ in range(args.steps):
        eager_step()
    torch.cuda.synchronize()
    prof = xm.xmoe_prof_read()
    # the shader clock the matrix-core kernels ran at in the last of these steps (the chip lowers it under this load;
    # the kernels sample it only while the launch profiler is on)
    clocks = xm.xmoe_prof_shader_clocks()
    xm.xmoe_prof_enable(False)
    xm.xmoe_prof_reset()

    flops, bytes_ = kernel_work(cfg, args.materialise_dy)
    small_bytes, f32_flops, small_mfma_flops = small_kernel_work(cfg)
    bytes_.update(small_bytes)
    gemm_work = GEMM_WORK_MLP2 if mlp2 else GEMM_WORK
    kernels = {}
    for name, (launches, total_ms) in prof.items():
        per_step_ms = total_ms / args.steps
        ent = {"launches_per_step": launches / args.steps, "ms_per_step": round(per_step_ms, 5),
               "avg_launch_us": round(total_ms * 1e3 / launches, 3)}
        if name in gemm_work:
            ent["tflops"] = round(flops[gemm_work[name]] / (per_step_ms * 1e-3) / 1e12, 3)
            ent["frac_mfma_peak"] = round(ent["tflops"] / PEAK_BF16_MFMA_TFLOPS, 5)
            ent["algorithmic_gbs"] = round(bytes_["gemm:" + gemm_work[name]] / (per_step_ms * 1e-3) / 1e9, 1)
        if name in small_mfma_flops:
            ent["tflops"] = round(small_mfma_flops[name] / (per_step_ms * 1e-3) / 1e12, 3)
            ent["frac_mfma_peak"] = round(ent["tflops"] / PEAK_BF16_MFMA_TFLOPS, 5)
        if name in f32_flops:
            ent["f32_tflops"] = round(f32_flops[name] / (per_step_ms * 1e-3) / 1e12, 3)
            ent["frac_f32_peak"] = round(ent["f32_tflops"] / PEAK_FP32_TFLOPS, 5)
        if name in clocks:
            ent["shader_clock_ghz"] = round(clocks[name], 3)
        if name in bytes_:
            ent["gbs"] = round(bytes_[name] / (per_step_ms * 1e-3) / 1e9, 2)
            ent["frac_hbm_peak"] = round(ent["gbs"] / PEAK_HBM_GBS, 5)
        kernels[name] = ent
    gemm_ms = sum(v["ms_per_step"] for n, v in kernels.items() if n in gemm_work)
    total_flops = sum(flops[k_] for k_ in (("up",) if mlp2 else ("gateup",)) + ("down", "dact", "dx", "wgrad"))
    dom = max((n for n in kernels if n in gemm_work), key=lambda n: kernels[n]["avg_launch_us"])
    dom_key = gemm_work[dom]
    # which roof binds the dominant kernel: the one that needs longer at its peak for the kernel's algorithmic work
    dom_flops = flops[dom_key] / kernels[dom]["launches_per_step"]
    dom_bytes = bytes_["gemm:" + dom_key] / kernels[dom]["launches_per_step"]
    dom_s = kernels[dom]["avg_launch_us"] * 1e-6
    hbm_bound = dom_bytes / (PEAK_HBM_GBS * 1e9) > dom_flops / (PEAK_BF16_MFMA_TFLOPS * 1e12)
    roofline = {
        "bound": "hbm" if hbm_bound else "mfma", "kernel": dom,
        "achieved": round(dom_bytes / dom_s / 1e9, 2) if hbm_bound else kernels[dom].get("tflops"),
        "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_MFMA_TFLOPS, "unit": "GB/s" if hbm_bound else "TFLOP/s",
        "frac": round(dom_bytes / dom_s / 1e9 / PEAK_HBM_GBS, 5) if hbm_bound
                else round(kernels[dom].get("tflops", 0.0) / PEAK_BF16_MFMA_TFLOPS, 5),
        "traffic": load_measured_traffic(cfg.name).get(dom),
        "flops_per_launch": dom_flops, "algorithmic_bytes_per_launch": dom_bytes,
        "frac_mfma_peak": round(dom_flops / dom_s / 1e12 / PEAK_BF16_MFMA_TFLOPS, 5),
        "frac_hbm_peak": round(dom_bytes / dom_s / 1e9 / PEAK_HBM_GBS, 5),
        "launches_per_step": kernels[dom]["launches_per_step"],
        "avg_launch_us": kernels[dom]["avg_launch_us"],
        "all_gemm_tflops": round(total_flops / (gemm_ms * 1e-3) / 1e12, 3),
        "all_gemm_frac": round(total_flops / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 5),
    }

    result = {
        "metric": "MoE-layer tokens/sec fwd+bwd at 1 GPU; grouped-GEMM % bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic", "launch": "hip graph" if args.graph else "eager",
        "config": {"workload": cfg.name, "expert": cfg.expert if not mlp2 else f"mlp2/{cfg.act}", "T": cfg.T, "d": cfg.d, "E": cfg.E, "E_s": cfg.E_s, "k": cfg.k, "f": cfg.f,
                   "rows_B": cfg.B, "skew_alpha": cfg.skew_alpha, "max_token_count": args.max_token_count, "useful_tflop_per_step": round(total_flops / 1e12, 4)},
        "fwd_only_ms": round(fwd_ms, 4),
        "fwd_only_tokens_per_s": round(cfg.T / (fwd_ms * 1e-3), 1),
        # what must survive from forward to backward for the routed rows: G and U (H for the two-matrix expert).  No
        # dispatched copy Xd (the gather is fused into the expert MLP's operand loads), no dY, and Y is read by the
        # forward combine only (the backward takes the combine weights' gradient from its own GEMM)
        "activation_bytes_held": sum(t_[:layer.B].numel() * t_.element_size()
                                     for t_ in (((layer.h,) if mlp2 else (layer.g, layer.u))
                                                + (() if layer.fuse_combine_bwd else (layer.y,)))),
        "layer_tflops": round(total_flops / (ms_per_step * 1e-3) / 1e12, 3),
        "grouped_gemm_pct_mfma_peak": round(100 * roofline["all_gemm_frac"], 3),
        "roofline": roofline,
        "hbm_copy_kernel_gbs": round(copy_gbs, 1),
        "vendor_dense_bf16_gemm_tflops": round(dense_tflops, 1),
        "kernels": kernels,
        "input_gen_s": round(t_gen, 1),
    }

    if args.rbd_experts_per_node > 0 and args.max_token_count is None:
        B, E = cfg.B, cfg.E
        i32 = dict(dtype=torch.int32, device="cuda")
        out = {n: torch.empty(B, **i32) for n in ("pilot_token_ids", "pilot_expert_ids", "replica_token_ids",
                                                  "replica_expert_ids", "s1_mapping_indices", "s1_mapping_experts",
                                                  "merge_src")}
        out.update({n: torch.empty(E, **i32) for n in ("pilot_tokens_per_expert", "replica_tokens_per_expert")})
        out.update({n: torch.empty(E + 1, **i32) for n in ("pilot_offsets", "replica_offsets")})
        keys = torch.from_numpy(xi.make_rbd_keys(B, cfg.seed).view(np.int32).copy()).cuda()
        ws_rbd = xm.alloc_workspace(xm.xmoe_workspace_bytes(xm.WS_RBD_STAGE0, cfg.T, cfg.d, E, cfg.k, cfg.f, 1))
        tok, eid = layer.token_ids[:B].contiguous(), layer.expert_ids
        off = layer.expert_offsets[:E + 1].contiguous()

        def rbd():
            xm.xmoe_rbd_stage0(layer.topk_idx, keys, tok, eid, off, layer.row_of_slot, args.rbd_experts_per_node, out,
                               ws_rbd)
        for _ in range(3):
            rbd()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            rbd()
        e1.record()
        torch.cuda.synchronize()
        n_pilot = int(out["pilot_offsets"][-1].item())
        result["rbd_stage0"] = {"experts_per_node": args.rbd_experts_per_node,
                                "us_per_call": round(e0.elapsed_time(e1) * 1e3 / args.steps, 2),
                                "pilots": n_pilot, "replicas": B - n_pilot,
                                "redundancy": round((B - n_pilot) / B, 4)}

    if not args.no_cpu_baseline:
        base, ref = cpu_baseline(cfg, args.cpu_sample_tokens, x_np, dout_np, wr_np, bias_np)
        result["cpu_baseline"] = base
        # parity of this very run: when the oracle's sample was the whole batch (and nothing was dropped), the step's
        # out and dx against it, in the figures of the whole-layer criterion
        criterion = ("max relative error 1e-5 element-wise" if cfg.dtype == "f32" else
                     "bf16 whole layer (about 8 bf16-stored intermediates between the unrounded float64 oracle and the "
                     "result): every output row's relative error in the 2-norm <= 2e-2 and every element's error "
                     "relative to max(|ref|, row RMS) <= 8e-2; single entry points hold 2e-2 element-wise")
        result["parity"] = {"criterion": criterion}
        if ref is not None and args.max_token_count is None:
            step()
            torch.cuda.synchronize()
            result["parity"]["out_row_elem"] = parity_against(ref[0], layer.out.float().cpu().numpy().astype(np.float64))
            result["parity"]["dx_row_elem"] = parity_against(ref[1], layer.dx.float().cpu().numpy().astype(np.float64))
    print(json.dumps(result))


def cpu_baseline(cfg, sample_tokens, x_np, dout_np, wr_np, bias_np):
    """The CPU oracle, as it stands, on the first `sample_tokens` tokens of the same workload (all experts'
    weights, forward + backward); tokens/s of that run."""
    import numpy as np

    import oracle
    import xmoe_inputs as xi
    Ts = min(sample_tokens, cfg.T)
    if cfg.expert == "mlp2":
        inp = {"x": x_np[:Ts], "dout": dout_np[:Ts], "w_router": wr_np, "bias": bias_np,
               "w1": xi.make_expert_weights(cfg, "w1"), "w2": xi.make_expert_weights(cfg, "w2")}
        t0 = time.perf_counter()
        fwd = oracle.moe2_layer_fwd(inp, cfg.k, cfg.act)
        bwd = oracle.moe2_layer_bwd(inp, fwd, cfg.k, cfg.act)
        dt = time.perf_counter() - t0
        return ({"value": round(Ts / dt, 2), "unit": "tokens/s", "cores": int(os.cpu_count()), "kind": "oracle",
                 "sample": f"first {Ts} of {cfg.T} tokens of workload {cfg.name}, all expert weights, fwd+bwd, "
                           f"float64 numpy, {dt:.1f} s"}, (fwd["out"], bwd["dx"]) if Ts == cfg.T else None)
    inp = {"x": x_np[:Ts], "dout": dout_np[:Ts], "w_router": wr_np, "bias": bias_np,
           "wg": xi.make_expert_weights(cfg, "wg"), "wu": xi.make_expert_weights(cfg, "wu"),
           "wd": xi.make_expert_weights(cfg, "wd"),
           "shared_wg": xi.make_shared_weights(cfg, "wg"), "shared_wu": xi.make_shared_weights(cfg, "wu"),
           "shared_wd": xi.make_shared_weights(cfg, "wd")}
    threads = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        nt = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        if nt:
            threads = max(nt)
    except Exception:
        pass
    t0 = time.perf_counter()
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    dt = time.perf_counter() - t0
    return ({"value": round(Ts / dt, 2), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
             "sample": f"first {Ts} of {cfg.T} tokens of workload {cfg.name}, all expert weights, fwd+bwd, "
                       f"float64 numpy, {dt:.1f} s"}, (fwd["out"], bwd["dx"]) if Ts == cfg.T else None)


if __name__ == "__main__":
    main()
