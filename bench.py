#!/usr/bin/env python3
"""Throughput of the OAPL loss head on one MI355X.

A step is one pass of the whole hot path (one oapl_loss_fwd_bwd call: log-prob
scoring, per-rollout sums, group value estimate, loss, backward to dH and dW)
over one synthetic batch of the Qwen-7B-shaped configuration (d = 4096,
V = 151936, 8 prompts x 8 rollouts, truncated-lognormal lengths).  Inputs are
resident in HBM before the timed region starts.

Prints one JSON line: rollout tokens/s, the roofline figures of the dominant
kernel (timed with HIP events on its own stream, inside the library), and the
CPU oracle timed on a bounded sample of the same batch on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz

# HBM bytes per launch of the dense kernels on the qwen7b workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE) scaled by what the same counters read for an elementwise kernel that
# moves 1 GiB each way (fetch x2.000, write x1.000); summary in profiles/traffic_qwen7b_fetch_write.txt.
# Valid only for the kernel sources they were taken with: the digest below is compared with the
# sources at run time and the figure is reported as null when they differ.
TRAFFIC = {
    "workload": "qwen7b",
    "sources_sha256_16": "1e30c9e65a5b3746",
    "per_launch_bytes": {          # averages over the step's 12 panels (11 of 12288 rows, one of 5729)
        "k_sweep": {"read": 17.34e9, "write": 7.17e9},
        "k_bwd_dh": {"read": 16.84e9, "write": 0.10e9},
        "k_bwd_dw": {"read": 19.40e9, "write": 2.49e9},
    },
}


def sources_digest():
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2602_19362_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen7b", help="name in synth.CONFIGS")
    ap.add_argument("--path", choices=["loss", "grpo", "logprob", "logprob_entropy", "sample"], default="loss",
                    help="loss: the whole hot path (default). logprob / logprob_entropy: oapl_logprob_fwd alone, "
                         "without / with the policy-entropy output (forward scoring only). "
                         "sample: oapl_sample_tokens (Gumbel-max draws at the workload's token temperature)")
    ap.add_argument("--panel-rows", type=int, default=0,
                    help="size the workspace for backward panels of at most this many token rows (0 = the "
                         "library's default); the library derives its panel from the workspace it is handed")
    ap.add_argument("--hidden-scale", type=float, default=1.0,
                    help="power probe, not a benchmark: multiply the hidden states by this before the run (0 = all-zero "
                         "H: same kernels, shapes and launch configuration, operands that toggle few bits); the JSON "
                         "line is marked and carries no baseline")
    ap.add_argument("--library-gemm-context", action="store_true",
                    help="context, not a benchmark: time the vendor library's bf16 GEMM (torch.matmul) on the three "
                         "contractions of one backward panel of the workload (scores, dH, dW; same H, W and a soft-max "
                         "panel computed from them), then exit; honours --hidden-scale")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, run a plain elementwise kernel that reads 1 GiB and writes 1 GiB "
                         "(the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def cpu_baseline(batch, n_tokens):
    """The oracle as it stands, on the first rollouts of the batch cut to n_tokens in all."""
    import numpy as np
    import torch
    from oracle import oapl_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    off = batch.seq_offsets.cpu().numpy()
    lens = np.diff(off)
    G = batch.cfg.n_rollouts
    per = max(1, n_tokens // G)
    take = np.minimum(lens[:G], per)                 # the first prompt's G rollouts, each cut to `per` tokens
    rows = np.concatenate([np.arange(off[s], off[s] + take[s]) for s in range(G)])
    f64 = lambda t: t.detach().cpu().to(torch.float64).numpy()
    rows_t = torch.from_numpy(rows).to(batch.H.device)
    H = f64(batch.H[rows_t])
    W = f64(batch.W)
    tok = batch.tokens[rows_t].cpu().numpy()
    logq = f64(batch.logq[rows_t])
    offs = np.concatenate([[0], np.cumsum(take)])
    t0 = time.perf_counter()
    orc.oapl_forward_backward(H, W, tok, logq, offs, f64(batch.rewards[:G]), np.zeros(G, dtype=np.int64), 1,
                              batch.beta, backward=batch.cfg.backward)
    dt = time.perf_counter() - t0
    return {
        "value": float(len(rows) / dt), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"first prompt's {G} rollouts cut to {per} tokens each ({len(rows)} tokens), "
                  f"fp64 numpy, forward{'+backward' if batch.cfg.backward else ''}, {dt:.1f} s",
    }


def library_gemm_context(torch, batch, cfg, args):
    """What the vendor library reaches on the same operands and shapes: the three dense contractions of
    one 12288-row panel as plain GEMMs (bf16 in, bf16 out, no soft-max, no accumulation into dW).  Says how
    much of the distance to the MFMA peak belongs to the chip (clock under load, operand delivery) rather
    than to the kernels here; it is not part of the measured path."""
    Tp = min(12288, batch.T)
    H, W = batch.H[:Tp].contiguous(), batch.W
    Z = torch.matmul(H, W.t())
    G = torch.softmax(Z.float(), dim=1)
    G[torch.arange(Tp, device=H.device), batch.tokens[:Tp].long()] -= 1.0
    G = G.to(torch.bfloat16)
    dH = torch.empty_like(H)
    dW = torch.empty_like(W)
    flop = 2.0 * Tp * cfg.V * cfg.d
    rows = []
    for name, fn in (("scores = H W^T", lambda: torch.matmul(H, W.t(), out=Z)),
                     ("dH = G W", lambda: torch.matmul(G, W, out=dH)),
                     ("dW = G^T H", lambda: torch.matmul(G.t(), H, out=dW))):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        rows.append({"gemm": name, "ms": round(ms, 3), "tflops": round(flop / ms / 1e9, 1),
                     "frac_of_bf16_peak": round(flop / ms / 1e9 / PEAK_BF16_TFLOPS, 4)})
    print(json.dumps({"context": "library_gemm", "workload": args.workload, "panel_rows": Tp, "d": cfg.d, "V": cfg.V,
                      "hidden_scale": args.hidden_scale, "launches_timed": args.steps, "gemms": rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path is built and measured single-GPU only "
              "(no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_19362_amd import oapl
    from workloads import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback of the product path)", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS[args.workload]
    batch = synth.make_batch(cfg, dev)
    T, d, V = batch.T, cfg.d, cfg.V
    if args.hidden_scale != 1.0:
        batch.H.mul_(args.hidden_scale)
    if args.library_gemm_context:
        library_gemm_context(torch, batch, cfg, args)
        return
    dt_code = oapl.OAPL_BF16 if cfg.dtype == "bf16" else oapl.OAPL_F32
    # the trainer knows its generation limit: panel buffers for the longest rollout of the workload
    longest = int((batch.seq_offsets[1:] - batch.seq_offsets[:-1]).max().item()) if batch.n_seq else 0
    ws_bytes, panel_rows, panel_buffers = oapl.workspace_bytes_for(T, d, V, batch.n_seq, batch.n_groups, dt_code,
                                                                   cfg.backward, args.panel_rows, longest)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    dH = torch.empty_like(batch.H) if cfg.backward else None
    dW = torch.empty((V, d), dtype=torch.float32, device=dev) if cfg.backward else None

    backward = cfg.backward and args.path in ("loss", "grpo")
    if args.path == "grpo":       # previous-policy log-probs: the engine's plus a small seeded lag
        g = torch.Generator(device=dev)
        g.manual_seed(synth.BASE_SEED + 977)
        logp_old = (batch.logq + 0.05 * torch.randn(T, generator=g, device=dev)).contiguous()

    def step():
        if args.path == "grpo":
            return oapl.grpo_loss_fwd_bwd(batch.H, batch.W, batch.tokens, batch.logq, logp_old, batch.seq_offsets,
                                          batch.rewards, batch.group_ids, batch.n_groups, backward=cfg.backward,
                                          workspace=ws, dH=dH, dW=dW)
        if args.path == "sample":
            return oapl.sample_tokens(batch.H, batch.W, cfg.token_temp, 2026, workspace=ws)
        if args.path != "loss":
            return oapl.logprob_fwd(batch.H, batch.W, batch.tokens, want_entropy=args.path == "logprob_entropy",
                                    workspace=ws)
        return oapl.loss_fwd_bwd(batch.H, batch.W, batch.tokens, batch.logq, batch.seq_offsets, batch.rewards,
                                 batch.group_ids, batch.n_groups, batch.beta, backward=cfg.backward,
                                 workspace=ws, dH=dH, dW=dW)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    oapl.timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kt = oapl.timing_read()
    oapl.timing_enable(False)
    status = oapl.read_device_status(ws)
    two_pass = bool(backward and oapl.took_two_passes(ws))
    loss = float(res.loss.item()) if args.path in ("loss", "grpo") else float(res[0].double().sum().item())
    # exact integer sums of the inputs' bit patterns: two runs that print the same digest computed on the same data
    inputs_digest = [int(batch.H.view(torch.int16).sum(dtype=torch.int64).item()),
                     int(batch.W.view(torch.int16).sum(dtype=torch.int64).item()),
                     int(batch.tokens.sum(dtype=torch.int64).item()),
                     int(batch.logq.view(torch.int32).sum(dtype=torch.int64).item())]
    if args.calibration_copy:
        x = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        y = torch.empty_like(x)
        for _ in range(3):
            torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y
    if status != 0 or loss != loss:
        print(f"device status {status}, loss {loss}", file=sys.stderr)
        sys.exit(1)

    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = T * args.steps / elapsed
    flop_unit = 2.0 * V * d                                  # one V x d contraction per token
    n_contractions = 3 if backward else 1                    # logits, dH, dW: what the method must compute
    alg_tflops = tokens_per_s * flop_unit * n_contractions / 1e12
    # executed: the single sweep visits the logits once (3 contractions); the two-pass schedule recomputes them (4)
    n_executed = (4 if two_pass else 3) if backward else 1
    hw_tflops = tokens_per_s * flop_unit * n_executed / 1e12

    # Each dense kernel executes 2*V*d flop per token it processes; over the
    # timed steps every kernel sees every token once per step.
    kernels = {}
    for name, (ms, n) in kt.items():
        if n == 0:
            continue
        tf = flop_unit * T * args.steps / (ms * 1e-3) / 1e12
        kernels[name] = {"launches": n, "avg_ms": ms / n, "tflops": tf, "frac": tf / PEAK_BF16_TFLOPS}
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches"]) if kernels else None
    roofline = None
    if dom:
        traffic = None
        if args.path == "loss" and args.workload == TRAFFIC["workload"] \
                and sources_digest() == TRAFFIC["sources_sha256_16"]:
            t = TRAFFIC["per_launch_bytes"].get(dom)
            traffic = None if t is None else t["read"] + t["write"]
        roofline = {"bound": "mfma", "kernel": dom, "achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": kernels[dom]["frac"], "traffic": traffic,
                    "avg_launch_ms": kernels[dom]["avg_ms"], "launches": kernels[dom]["launches"]}

    out = {
        "metric": "rollout tokens/s for OAPL logprob+loss fwd+bwd; % of bf16 MFMA peak" if args.path == "loss"
        else "rollout tokens/s for the GRPO baseline loss fwd+bwd on the same head" if args.path == "grpo" else f"rollout tokens/s for the forward-only entry point ({args.path}); % of bf16 MFMA peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: d={d} V={V} {cfg.n_prompts} prompts x {cfg.n_rollouts} rollouts, "
                               f"T={T} packed tokens, beta={cfg.beta}, {'fwd+bwd' if backward else 'fwd only'}"},
        "algorithmic_tflops": alg_tflops, "frac_of_bf16_peak_algorithmic": alg_tflops / PEAK_BF16_TFLOPS,
        "executed_tflops": hw_tflops, "frac_of_bf16_peak_executed": hw_tflops / PEAK_BF16_TFLOPS,
        "schedule": ("two_pass" if two_pass else "single_sweep") if backward else "forward_only",
        "workspace_bytes": ws_bytes, "panel_rows": panel_rows if backward else None,
        "panel_buffers": panel_buffers if backward else None, "longest_rollout": longest,
        "kernels": kernels, "roofline": roofline, "loss" if args.path in ("loss", "grpo") else "output_checksum": loss,
        "inputs_digest": inputs_digest,
    }
    if args.hidden_scale != 1.0:
        out["power_probe"] = f"hidden states scaled by {args.hidden_scale}: not the benchmark workload"
    if not args.no_cpu_baseline and args.path == "loss" and args.hidden_scale == 1.0:
        out["cpu_baseline"] = cpu_baseline(batch, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
