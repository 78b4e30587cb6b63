#!/usr/bin/env python3
"""Benchmark of the fused LM-head log-prob + policy-loss forward+backward on one MI355X.

One step = one call of rl_policy_loss_fwd_bwd (prep, forward, advantage, loss, backward) over
one seeded synthetic rollout batch that is already resident in HBM.  Prints ONE JSON line:
rollout tokens/s (mask=1 rows only), the MFMA roofline of the dominant contraction kernel
(timed live with HIP events on the library's stream) and the float64 oracle timed on the
host cores on a bounded token-sub-sampled sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3
# HBM-side bytes (L2 <-> fabric; FETCH_SIZE x2.0 + WRITE_SIZE x1.0 after calibration against a plain 1 GiB copy)
# of the largest launch of each contraction class on the default workload, from two rocprofv3 --pmc runs per
# backward mode whose summary is profiles/gemm_nt_bf16_7b.md.  Counters cannot be read live, so these are constants of that run.
MEASURED_TRAFFIC_7B = {        # default chunks: 40960 rows single-pass ("stash"), 32768 rows recompute
    "stash": {"gemm_fwd": 96.4e9 + 12.7e9, "gemm_bwd": 198.3e9 + 2.5e9},
    "recompute": {"gemm_fwd": 53.6e9 + 0.3e9, "gemm_ds": 57.4e9 + 10.0e9, "gemm_dx": 61.8e9 + 0.2e9, "gemm_dw": 85.1e9 + 2.2e9},
}
CPU_SAMPLE_LEN_DIV = {"tiny": 1, "small": 8, "7b": 160, "long": 640, "32b": 768}   # ~10-30 s of oracle work


def cpu_baseline(name: str, objective: str):
    """Time the oracle, as it stands, on a token-sub-sampled instance of the same workload."""
    import numpy as np
    import torch
    from oracle import policy_oracle as orc
    from paper_2603_16435_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    div = CPU_SAMPLE_LEN_DIV[name]
    b = synth.make_rollouts(name, "cpu", "packed", len_div=div)

    def bits(t):
        t = t.contiguous()
        return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.numpy()

    c = b.cfg
    t0 = time.perf_counter()
    orc.policy_loss_fwd_bwd(orc.GRPO if objective == "grpo" else orc.FLOW, bits(b.hidden), bits(b.weight),
                            bits(b.token_ids), bits(b.mask), bits(b.cu_seqlens), bits(b.group_idx), bits(b.rewards),
                            bits(b.old_logprob), bits(b.ref_logprob), bits(b.log_z), c.P, clip_eps=c.clip_eps,
                            kl_coef=c.kl_coef, beta=c.beta, adv_eps=c.adv_eps, adv_std_ddof=c.adv_std_ddof)
    dt = time.perf_counter() - t0
    return {"value": b.T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"same config, every sequence cut to ceil(len/{div}) tokens: {b.T} tokens, "
                      f"full H={c.H} V={c.V}, fwd+bwd in float64, {dt:.1f} s"}


def bench_logz_head(a, dev):
    """The log-Z head of the same configuration: P prompts of U[128,1024] hidden-state rows, M = H, forward + backward."""
    import numpy as np
    import torch
    from paper_2603_16435_amd import binding, synth
    cfg = synth.CONFIGS[a.config]
    P, H, M = cfg.P, cfg.H, cfg.H
    g = torch.Generator().manual_seed(cfg.seed)
    lens = torch.randint(128, 1025, (P,), generator=g)
    cu = torch.cat([torch.zeros(1, dtype=torch.int64), lens.cumsum(0)]).to(torch.int32).to(dev)
    rows = int(lens.sum())
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    X = torch.randn(rows, H, generator=g).to(dt).to(dev)
    W1 = (torch.randn(M, H, generator=g) / np.sqrt(H)).to(dev); b1 = torch.zeros(M, device=dev)
    w2 = (torch.randn(M, generator=g) / np.sqrt(M)).to(dev); b2 = torch.zeros(1, device=dev)
    d = torch.randn(P, generator=g).to(dev)
    _, ws = binding.rl_logz_head_forward(X, cu, W1, b1, w2, b2)

    def step():
        binding.rl_logz_head_forward(X, cu, W1, b1, w2, b2, workspace=ws)
        binding.rl_logz_head_backward(d, w2, H, ws)
    for _ in range(max(a.warmup, 1)):
        step()
    torch.cuda.synchronize()
    steps = max(a.steps, 20)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    # bytes the head must move: prompt rows once, W1 read once, dW1 written once (activations are a few hundred KB)
    algo = rows * H * X.element_size() + 4.0 * M * H + 4.0 * M * H
    out = {"metric": "log-Z head forward+backward, prompts/s", "value": P / sec, "unit": "prompts/s", "n_gpus": 1, "steps": steps,
           "warmup": max(a.warmup, 1), "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"log-Z head of {a.config}: P={P} prompts, {rows} prompt rows, H={H}, hidden units M={M}, {cfg.dtype} states, f32 parameters"},
           "roofline": {"bound": "hbm", "achieved": algo / sec / 1e9, "peak": 8000.0, "unit": "GB/s", "frac": algo / sec / 8e12, "traffic": None,
                        "note": "five small launches per step plus host-side marshalling: launch-latency-bound at this size (W1 and dW1 are 51 MB each)"}}
    print(json.dumps(out), flush=True)


def bench_rvq_encode(a, dev):
    """Residual-VQ encode of one local window of key-cache vectors in the paper's 8B setting: N = 56 codebooks of
    S = 1024 entries, D = 128, L = 1024 vectors per (layer, head) group; 128 groups per call here (two workgroups per CU)."""
    import numpy as np
    import torch
    from paper_2603_16435_amd import binding, synth
    G, L, N, S, D = 128, 1024, 56, 1024, 128
    x, cb = synth.make_rvq_case(G, L, N, S, D, device=dev)
    norms = binding.rl_rvq_codebook_norms(cb)
    for _ in range(max(a.warmup, 1)):
        binding.rl_rvq_encode(x, cb, norms)
    torch.cuda.synchronize()
    steps = max(a.steps, 5)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        codes, res = binding.rl_rvq_encode(x, cb, norms)
    e1.record(); torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / steps
    flops = 2.0 * G * L * S * D * N
    out = {"metric": "residual-VQ encode, vectors/s", "value": G * L / sec, "unit": "vectors/s", "n_gpus": 1, "steps": steps,
           "warmup": max(a.warmup, 1), "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"key-cache window of the paper's 8B setting: G={G} groups x L={L} vectors, D={D}, N={N} stages of S={S} entries "
                                  "(synthetic Gaussian codebooks; no trained ones exist here)"},
           "roofline": {"bound": "mfma", "kernel": "rvq_encode_kernel", "achieved": flops / sec / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": flops / sec / 1e12 / PEAK_BF16_TFLOPS, "traffic": 3.2e9,
                        "traffic_note": "rocprofv3 FETCH_SIZE of one launch, scaled x2.0 (profiles/rvq_encode_8b_key.md); the 0.06 GB of codes and residuals written are not in it",
                        "note": "2 L S D N flop per group; with K = D = 128 every MFMA needs eleven issue cycles of arg-max bookkeeping on the same port: "
                                "issue-bound, not power-bound (profiles/rvq_encode_8b_key.md)"}}
    if not a.no_cpu_baseline:
        from oracle import rvq_oracle as rvq
        t0 = time.perf_counter()
        for gi in range(2):
            xs = x[gi].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            cbs = cb[gi].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            rvq.rvq_encode(xs, cbs)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * L / dt, "unit": "vectors/s", "cores": 1, "kind": "oracle",
                               "sample": f"groups 0 and 1 ({2 * L} vectors), all {N} stages, float64, {dt:.1f} s"}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="7b", choices=["tiny", "small", "7b", "long", "32b"])
    ap.add_argument("--objective", default="grpo", choices=["grpo", "flow"])
    ap.add_argument("--layout", default="padded", choices=["padded", "packed"])
    ap.add_argument("--chunk-rows", type=int, default=0)
    ap.add_argument("--backward", default="auto", choices=["auto", "recompute", "stash"],
                    help="backward mode of the library; auto = single-pass (stash) with max_seq_len = the config's longest response")
    ap.add_argument("--len-div", type=int, default=1, help="shorten every sequence (debug / profiling runs)")
    ap.add_argument("--path", default="policy-loss", choices=["policy-loss", "logz-head", "rvq-encode"],
                    help="logz-head: time the small upstream head (forward + backward) instead of the hot path")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="time only the headline (objective, backward) pair, not the other objective and the recompute backward")
    ap.add_argument("--secondary-steps", type=int, default=5, help="timed steps of each secondary measurement (3 warm-ups each)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run one plain 1 GiB device copy (reference dispatch for FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. "
              "Sharding is design-only (whole prompts per GPU, or vocab-parallel W).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_16435_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if a.path == "logz-head":
        return bench_logz_head(a, dev)
    if a.path == "rvq-encode":
        return bench_rvq_encode(a, dev)
    b = synth.make_rollouts(a.config, dev, a.layout, len_div=a.len_div)
    cfg = b.cfg
    batch = binding.make_batch(b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens, b.group_idx, b.rewards,
                               b.old_logprob, b.ref_logprob, b.log_z, cfg.P)

    # headline: the objective and backward mode asked for (default: GRPO, auto = single pass)
    head = time_mode(a, b, batch, a.objective, a.backward, a.steps, a.warmup)

    # what a pure MFMA loop with toggling random operands reaches on this part right now (no memory traffic)
    peak_burst = binding.rl_measure_mfma_peak(200, dev)
    peak_sustained = binding.rl_measure_mfma_peak(1000, dev)

    # the other half of the target, timed the same way in the same run: the other objective in the same mode, and the
    # backward that recomputes the logits tile by tile (the problem statement's wording; four contractions instead of three)
    secondary = {}
    if not a.no_secondary:
        other = "flow" if a.objective == "grpo" else "grpo"
        for key, objective, backward in ((f"{other}_{a.backward}", other, a.backward),
                                         (f"{a.objective}_recompute", a.objective, "recompute"),
                                         (f"{other}_recompute", other, "recompute")):
            if (backward == a.backward and objective == a.objective) or key in secondary:
                continue
            r = time_mode(a, b, batch, objective, backward, a.secondary_steps, 3)
            secondary[key] = {k: r[k] for k in ("objective", "backward", "backward_resolved", "steps", "warmup", "value", "unit",
                                                 "ms_per_step", "ms_per_step_median", "ms_per_step_min", "mfma_frac_6THV",
                                                 "tflops_6THV", "roofline", "loss")}
            secondary[key]["class_ms_per_step"] = {k: round(v["ms_per_step"], 3) for k, v in r["kernels"].items() if v["ms_per_step"] > 0}
            secondary[key]["class_tflops"] = {k: round(v["tflops"], 1) for k, v in r["kernels"].items() if v["tflops"]}

    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    T = head["T"]
    achieved = head["roofline"]["achieved"]
    out = {
        "metric": "rollout tokens/sec, fused logprob+policy-loss fwd+bwd; % bf16 MFMA peak",
        "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"], "ms_per_step_min": head["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{a.config}: P={cfg.P} G={cfg.G} len U[{cfg.len_lo},{cfg.len_hi}] H={cfg.H} V={cfg.V} "
                               f"{cfg.dtype}, {a.layout} rows R={b.R}, real tokens T={T}, objective={a.objective}, "
                               f"backward={head['backward_resolved']}"
                               + (f", len_div={a.len_div}" if a.len_div != 1 else ""),
                   "objective": a.objective, "layout": a.layout, "T": T, "R": b.R, "H": cfg.H, "V": cfg.V,
                   "chunk_rows": head["chunk_rows"], "backward": a.backward, "backward_resolved": head["backward_resolved"]},
        "mfma_frac_6THV": head["mfma_frac_6THV"],
        "tflops_6THV": head["tflops_6THV"],
        "roofline": head["roofline"],
        "mfma_only_measured": {"burst_200ms": {"tflops": peak_burst[0], "shader_mhz": peak_burst[1]},
                               "sustained_1s": {"tflops": peak_sustained[0], "shader_mhz": peak_sustained[1]},
                               "roofline_frac_of_sustained": achieved / peak_sustained[0] if peak_sustained[0] > 0 else None},
        "kernels": head["kernels"],
        "hbm_bound_classes": head["hbm_bound_classes"],
        "loss": head["loss"],
        "secondary": secondary,
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.config, a.objective)
    print(json.dumps(out), flush=True)


def time_mode(a, b, batch, objective: str, backward: str, steps: int, warmup: int) -> dict:
    """`warmup` untimed and `steps` timed calls of rl_policy_loss_fwd_bwd for one objective and backward mode, between
    synchronisations; per-class launch times from HIP events the library records on its own stream."""
    import torch
    from paper_2603_16435_amd import binding
    cfg = b.cfg
    dev = b.hidden.device
    obj = binding.OBJECTIVES[objective]
    prm = binding.make_params(cfg.clip_eps, cfg.kl_coef, cfg.beta, cfg.adv_eps, cfg.adv_std_ddof, a.chunk_rows,
                              backward_mode=backward, max_seq_len=int(b.lengths.max()))
    plan = binding.PolicyLossPlan(batch, prm, dev, b.hidden.dtype, backward=True)
    for _ in range(warmup):
        plan.run(obj)
    torch.cuda.synchronize()
    binding.rl_profile_enable(True)
    binding.rl_profile_read()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # on the stream the library launches on
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        res = plan.run(obj)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    prof = binding.rl_profile_read()
    binding.rl_profile_enable(False)

    # launches per step that have rows to work on (the library launches a fixed upper bound of chunks; the rest return at once)
    stash = prof["gemm_bwd"][1] > 0
    default_tc = binding.lib().rl_default_chunk_rows_single_pass() if stash else binding.lib().rl_default_chunk_rows()
    tc = a.chunk_rows or default_tc
    if stash:                                  # sequence-aligned chunks: greedy packing of whole sequences
        real_chunks, rows = 1, 0
        for n in b.lengths.tolist():
            if rows > 0 and rows + n > tc:
                real_chunks, rows = real_chunks + 1, 0
            rows += n
    else:
        real_chunks = -(-b.T // tc)
    st = res.stats_dict()
    T = int(st["n_tokens"])
    loss = float(res.loss.item())
    assert T == b.T and loss == loss and st["n_overflow_rows"] == 0, (T, b.T, loss, st)
    thv = float(T) * cfg.H * cfg.V
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    # dominant kernel: the contraction class with the largest share of the step
    # flops of one step per launch class: each contraction is 2*T*H*V; gemm_bwd is dX and dW in one launch
    class_flops = {"gemm_fwd": 2.0 * thv, "gemm_ds": 2.0 * thv, "gemm_dx": 2.0 * thv, "gemm_dw": 2.0 * thv, "gemm_bwd": 4.0 * thv}
    gemms = {k: prof[k] for k in class_flops}
    dom = max(gemms, key=lambda k: gemms[k][0])
    dom_ms, dom_n = gemms[dom]
    achieved = class_flops[dom] * steps / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    kernels = {k: {"ms_per_step": v[0] / steps, "launches_per_step": v[1] / steps,
                   "tflops": (class_flops[k] * steps / (v[0] * 1e-3) / 1e12) if (k in gemms and v[0] > 0) else None}
               for k, v in prof.items()}
    # The O(T) launch classes against the HBM roofline: algorithmic bytes per step (what the stage must read and
    # write once, from the shapes) / event-timed duration.  They are launch-latency-bound at these sizes.
    esz = 2 if cfg.dtype == "bf16" else 4
    tiles_v = -(-cfg.V // 256)
    R, Hh, Vv = b.R, cfg.H, cfg.V
    class_bytes = {
        # mask + ids read, three zero-filled row outputs + compaction index, compacted ids / row map written;
        # single pass also reads each token's x row and W[y] row for the target logit
        "prep": R * (1 + 4 + 12 + 4) + T * 8 + (T * 2 * Hh * esz if stash else 0),
        # per-tile partials (float2 single pass, float4 recompute) in, lse / logp / entropy out
        "combine": tiles_v * T * (8 if stash else 16) + T * 24,
        # logp, old, ref, row map in; c_t twice out; single pass: the per-row patch and factor as well
        "loss": T * 24 + (T * 26 if stash else 0),
        # W -> W^T and the X chunks -> X^T (read + write), masked dX rows zeroed
        "transpose": 2 * Vv * Hh * esz + 2 * T * Hh * esz + (R - T) * Hh * esz,
    }
    hbm = {}
    for k, nbytes in class_bytes.items():
        ms = prof[k][0] / steps
        if ms > 0:
            gbps = nbytes / (ms * 1e-3) / 1e9
            hbm[k] = {"ms_per_step": ms, "algorithmic_bytes_per_step": nbytes, "gbps": gbps, "frac_of_8TBps": gbps / 8000.0}
    mode_key = "stash" if stash else "recompute"
    kernel_name = {"gemm_fwd": "gemm_nt_bf16_kernel<EpiFwdStash>" if stash else "gemm_nt_bf16_kernel<EpiFwd>",
                   "gemm_ds": "gemm_nt_bf16_kernel<EpiDS>", "gemm_dx": "gemm_nt_bf16_kernel<EpiDX>",
                   "gemm_dw": "gemm_nt_bf16_kernel<EpiDW>", "gemm_bwd": "gemm_nt_bf16_pair_kernel<EpiDX, EpiDW>"}[dom]
    out = {
        "objective": objective, "backward": backward, "backward_resolved": "single-pass" if stash else "recompute",
        "steps": steps, "warmup": warmup, "T": T, "chunk_rows": tc,
        "value": T * steps / dt, "unit": "tokens/s",
        "ms_per_step": dt / steps * 1e3, "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
        "mfma_frac_6THV": 6.0 * thv / (dt / steps) / 1e12 / peak,
        "tflops_6THV": 6.0 * thv / (dt / steps) / 1e12,
        "roofline": {"bound": "mfma", "kernel": f"{kernel_name} ({dom})", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": (MEASURED_TRAFFIC_7B[mode_key].get(dom)
                                 if (a.config == "7b" and a.len_div == 1 and a.layout == "padded"
                                     and tc == default_tc) else None),
                     "traffic_note": "HBM-side bytes of the largest launch of this class (rocprofv3 FETCH_SIZE/WRITE_SIZE, profiles/gemm_nt_bf16_7b.md)",
                     "launches_with_work": real_chunks * steps, "launches": int(dom_n),
                     "avg_launch_ms": dom_ms / max(real_chunks * steps, 1),
                     "flops_per_avg_launch": class_flops[dom] / real_chunks},
        "kernels": kernels,
        "hbm_bound_classes": hbm,
        "loss": loss,
    }
    del plan, res
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
