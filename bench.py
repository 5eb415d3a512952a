#!/usr/bin/env python3
"""Benchmark of the HiFT step on one MI355X.

A "step" is one pass of the whole hot path (forward over all units, truncated backward, weight
gradients and optimizer update of the active group, optimizer-state movement) over one batch.
Workload: the LLaMA-7B-shaped decoder, batch 4 x 512 tokens, m = 1 (34 groups), bottom2up,
AdamW, optimizer state of inactive groups in pinned host memory.  Tokens are bounded Zipf(1.1),
weights N(0, 0.02^2): synthetic stand-ins, resident in HBM before the timed region starts.

Prints one JSON line: trained tokens/s over the timed steps, the MFMA roofline figures of the
linear-layer contraction class measured with HIP events inside the timed region, and the CPU
oracle timed on this machine's host cores on a bounded sample (the same widths at depth 2).
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

import numpy as np  # noqa: E402

BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA


def cpu_baseline(wl_name, seed):
    """Times one oracle step on the depth-2 twin of the workload (same widths, batch, sequence)."""
    from hift_inputs import WORKLOADS, init_params, make_batch, model_config
    from oracle import hift_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    full, twin = WORKLOADS[wl_name], WORKLOADS[wl_name + "_L2"]
    cfg = model_config(twin)
    spec = [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]
    theta = init_params(seed, spec, bf16_exact=True).astype(np.float64)
    orc = O.HiftOracle(cfg, twin["opt"], theta, half_weights=True)
    orc.set_group_schedule("bottom2up", 1, 0)
    tok, lab = make_batch(twin, seed, 1)
    t0 = time.perf_counter()
    orc.step(tok, lab, 1)
    dt = time.perf_counter() - t0
    T = tok.size
    # matrix-product flops of a full (untruncated) step: 6 per parameter of the linear layers
    # per token, plus attention; the oracle always does the full backward
    def step_flops(L):
        c = model_config(full, n_layers=L)
        d, f, V, S = c["d_model"], c["d_ffn"], c["vocab"], twin["seq"]
        layer = 4 * d * d + 3 * d * f
        att = 2 * 2 * S * d
        return 3.0 * T * (2 * L * layer + L * att + 2 * V * d)
    scale = step_flops(full["n_layers"]) / step_flops(2)
    return {
        "value": T / (dt * scale), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"one float64 oracle step (full forward and backward, AdamW on one layer) on the depth-2 twin "
                   f"of {wl_name} (same widths, batch {twin['batch']} x {twin['seq']}): {dt:.1f} s = {T / dt:.1f} tokens/s; "
                   f"value is that rate scaled to {full['n_layers']} layers by the matrix-product flop ratio {scale:.2f}"),
    }


HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E


def hbm_rooflines(rowwise, n_opt, ms_opt, by_opt, n_pack, ms_pack, by_pack):
    """Achieved GB/s against the 8 TB/s peak for every memory-bound kernel kind that ran in the event-bracketed
    pass: algorithmic bytes (each element read once, each written once) / event time."""
    out = {}
    rows = dict(rowwise)
    rows["optimizer update (one entry per step)"] = (n_opt, ms_opt, by_opt)
    rows["weight re-pack (one entry per step)"] = (n_pack, ms_pack, by_pack)
    for name, (n, ms, b) in rows.items():
        if n == 0 or ms <= 0:
            continue
        gbps = b / (ms * 1e-3) / 1e9
        out[name] = {"launches": n, "avg_us": round(1e3 * ms / n, 2), "mb_per_launch": round(b / n / 1e6, 2),
                     "gbps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 3)}
    return out


def measured_traffic():
    """HBM bytes per launch of the dominant kernel from the committed counter runs, or None when
    the kernel source has changed since they were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    src = os.path.join(ROOT, "paper_2401_15207_amd", "csrc", "gemm.hip")
    try:
        rec = json.load(open(path))
        if rec.get("gemm_hip_sha256") != hashlib.sha256(open(src, "rb").read()).hexdigest():
            return None
        return rec["hbm_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        return None


def kernel_bench(reps, n_weights=1, vendor=False, ksweep=False):
    """Times the linear-layer contraction at every shape of the 7B workload, stand-alone, with
    HIP events on the launch stream, then runs one plain 1 GiB device copy (the reference
    kernel for scaling hardware byte counters).  One JSON line.

    n_weights: how many copies of the weight operand the launches of a shape rotate through.  With one, the
    operand stays in the last-level cache from launch to launch; inside a training step every weight is read once
    per pass and comes from HBM, which 8 copies reproduce.  vendor: also time the same products through
    torch.matmul (the vendor library's kernels), launches interleaved in the same process; its dW product writes
    bf16 where this library's writes fp32."""
    import torch
    import paper_2401_15207_amd as H
    T, d, f, V = 2048, 4096, 11008, 32000
    shapes = [  # name, M, N, K, a_kmajor, b_kmajor, out_f32
        ("fwd_qkv", T, 3 * d, d, 1, 1, 0), ("fwd_o", T, d, d, 1, 1, 0), ("fwd_gate_up", T, 2 * f, d, 1, 1, 0),
        ("fwd_down", T, d, f, 1, 1, 0), ("fwd_head", T, V, d, 1, 1, 0),
        ("dx_qkv", T, d, 3 * d, 1, 0, 0), ("dx_o", T, d, d, 1, 0, 0), ("dx_gate_up", T, d, 2 * f, 1, 0, 0),
        ("dx_down", T, f, d, 1, 0, 0), ("dx_head", T, d, V, 1, 0, 0),
        ("dw_qkv", 3 * d, d, T, 0, 0, 1), ("dw_o", d, d, T, 0, 0, 1), ("dw_gate_up", 2 * f, d, T, 0, 0, 1),
        ("dw_down", d, f, T, 0, 0, 1), ("dw_head", V, d, T, 0, 0, 1),
    ]
    if ksweep:  # one round of 128 x 256 tiles at growing K: the fixed cost of a round is the intercept
        shapes = [("k%d" % K, T, d, K, 1, 1, 0) for K in (256, 512, 1024, 2048, 4096, 8192)]
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    out = {}
    st = torch.cuda.current_stream()
    ws = torch.zeros(H.kernel_packed_workspace_bytes() // 4, device="cuda", dtype=torch.float32)

    def timed(launch):
        for i in range(max(2, n_weights)):
            launch(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for i in range(reps):
            launch(i)
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    for name, M, N, K, ak, bk, of in shapes:
        A = (torch.randn(M * K, generator=g, device="cuda") * 0.5).to(torch.bfloat16)
        Bs = [(torch.randn(N * K, generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_weights)]
        C = torch.empty(M * N, device="cuda", dtype=torch.float32 if of else torch.bfloat16)
        lda, ldb = (K if ak else M), (K if bk else N)
        # forward and dX multiply by a weight matrix: the model keeps those in fragment order and runs the
        # packed-operand kernel (with its work space for a shared last round); dW has two activation operands
        # stored contraction-index first and runs gemm_tt_k
        packed = ak == 1 and H.kernel_packed_bytes(N, K) > 0
        if packed:
            Bps = []
            for B in Bs:
                Bp = torch.empty(H.kernel_packed_bytes(N, K) // 2, device="cuda", dtype=torch.bfloat16)
                H.kernel_pack_b(bk, N, K, B, ldb, Bp)
                Bps.append(Bp)
            launch = lambda i: H.kernel_gemm_packed_ws(of, M, N, K, A, lda, Bps[i % n_weights], C, N, None, None, ws)
        else:
            launch = lambda i: H.kernel_gemm(1, ak, bk, of, M, N, K, A, lda, Bs[i % n_weights], ldb, C, N)
        ms = timed(launch)
        alg_bytes = 2 * (M * K + N * K) + (4 if of else 2) * M * N
        out[name] = {"M": M, "N": N, "K": K, "us": 1e3 * ms, "tflops": 2.0 * M * N * K / ms / 1e9,
                     "algorithmic_bytes": alg_bytes, "weights_in_rotation": n_weights,
                     "kernel": "gemm_pk_k" if packed else ("gemm_tt_k" if not ak and not bk else "gemm_mfma_k")}
        if vendor:
            Am = A.view(M, K) if ak else A.view(K, M).t()
            Bms = [B.view(N, K).t() if bk else B.view(K, N) for B in Bs]
            Cv = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
            vms = timed(lambda i: torch.matmul(Am, Bms[i % n_weights], out=Cv))
            out[name]["vendor_us"] = 1e3 * vms
            out[name]["vendor_tflops"] = 2.0 * M * N * K / vms / 1e9
            del Am, Bms, Cv
        del A, Bs, C, launch
        if packed:
            del Bps
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)                      # plain copy kernel: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    print(json.dumps({"kernel_bench": out, "copy_reference_bytes_each_way": 1 << 30}))


def lora_bench(a):
    """The LoRA baseline of section 4.3 on the same kernels: adapters of rank --lora-rank on the query and value
    projections, full forward, activation gradients down to the first layer, AdamW on the adapters.  One JSON line
    (not the benchmark's metric: a comparison figure)."""
    import torch
    import paper_2401_15207_amd as H
    from hift_inputs import WORKLOADS, fill_weights_on_device, make_batch, model_config
    wl = WORKLOADS[a.workload]
    cfg = model_config(wl)
    B, S = wl["batch"], wl["seq"]
    model = H.HiftModel(cfg, wl["opt"], 1, B, S, init_params=None, lora_rank=a.lora_rank, lora_alpha=2.0 * a.lora_rank)
    fill_weights_on_device(model, a.seed)
    g = torch.Generator(device="cuda")
    g.manual_seed(a.seed + 1)
    model.lora_write((torch.randn(model.lora_param_count(), generator=g, device="cuda") * 0.02).cpu().numpy())
    n_total = a.steps + a.warmup
    batches = []
    for t in range(1, n_total + 1):
        tok, lab = make_batch(wl, a.seed, t)
        batches.append((torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()))
    for t in range(a.warmup):
        model.lora_step(*batches[t], want_loss=False)
    model.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(a.warmup, n_total):
        model.lora_step(*batches[t], want_loss=False)
    model.synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    model.profile_enable(True)
    for t in range(a.warmup, n_total):
        model.lora_step(*batches[t], want_loss=False)
    model.synchronize()
    cls = {name: model.profile_read(i)[1] / max(a.steps, 1) for i, name in
           enumerate(["linear_gemm_packed", "attention_gemm", "rowwise_elementwise", "optimizer", "linear_gemm_other", "weight_repack"])}
    model.profile_enable(False)
    loss = model.lora_step(*batches[0], want_loss=True)
    print(json.dumps({"lora_step": {"workload": a.workload, "rank": a.lora_rank, "adapter_params": model.lora_param_count(),
                                    "tokens_per_s": a.steps * B * S / elapsed, "ms_per_step": 1e3 * elapsed / max(a.steps, 1),
                                    "steps": a.steps, "warmup": a.warmup, "kernel_classes_ms_per_step": cls, "last_loss": loss,
                                    "memory_gb": round(model.memory()["total"] / 1e9, 2)}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=34)
    ap.add_argument("--warmup", type=int, default=34)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--copy-engine", type=int, default=0, help="0 hipMemcpyAsync, 1 small-grid copy kernel")
    ap.add_argument("--copy-blocks", type=int, default=16)
    ap.add_argument("--m", type=int, default=0,
                    help="units per group (default: the workload's); the number of units gives one group, "
                         "i.e. a full fine-tuning step on the same kernels")
    ap.add_argument("--state-resident", action="store_true", help="keep all optimizer state in HBM")
    ap.add_argument("--opt", default="", choices=["", "adamw", "adagrad", "sgdm", "sgd"],
                    help="optimizer (default: the workload's AdamW); the 13B-shaped workload sweeps them")
    ap.add_argument("--strategy", default="", choices=["", "bottom2up", "top2down", "random"])
    ap.add_argument("--master-on-host", action="store_true",
                    help="park the fp32 master of inactive groups in pinned memory too (small-memory mode)")
    ap.add_argument("--no-packed-copies", action="store_true",
                    help="do not keep the fragment-order weight copies (small-memory mode; slower contractions)")
    ap.add_argument("--lora-rank", type=int, default=0,
                    help="time the LoRA comparison step (adapters of this rank on the query and value projections) and exit")
    ap.add_argument("--kernel-bench", type=int, default=0, metavar="REPS",
                    help="time the contraction kernel alone at the 7B shapes, REPS launches each, and exit")
    ap.add_argument("--kernel-bench-weights", type=int, default=1, metavar="N",
                    help="with --kernel-bench: rotate each shape's launches through N copies of the weight operand "
                         "(8: the weights come from HBM as inside a step; 1: they stay in the last-level cache)")
    ap.add_argument("--kernel-bench-ksweep", action="store_true",
                    help="with --kernel-bench: instead of the 7B shapes, M = 2048, N = 4096 (one round of tiles) at K = 256 ... 8192")
    ap.add_argument("--vendor-library", action="store_true",
                    help="with --kernel-bench: also time the same products through torch.matmul")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: the HiFT step library is single-GPU in this build "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    if a.kernel_bench > 0:
        kernel_bench(a.kernel_bench, a.kernel_bench_weights, a.vendor_library, a.kernel_bench_ksweep)
        return
    if a.lora_rank > 0:
        lora_bench(a)
        return

    import torch
    import paper_2401_15207_amd as H
    from hift_inputs import WORKLOADS, fill_weights_on_device, make_batch, model_config

    wl = WORKLOADS[a.workload]
    cfg = model_config(wl)
    B, S = wl["batch"], wl["seq"]
    t_setup = time.perf_counter()
    if a.m > 0:
        wl = dict(wl, m=a.m)
    if a.opt:
        lr = wl["opt"]["lr"]
        wl = dict(wl, opt={"adamw": wl["opt"],
                           "adagrad": dict(kind="adagrad", lr=lr, eps=1e-10, weight_decay=0.0, momentum=0.0),
                           "sgdm": dict(kind="sgd", lr=lr, momentum=0.9, weight_decay=0.0),
                           "sgd": dict(kind="sgd", lr=lr, momentum=0.0, weight_decay=0.0)}[a.opt])
    if a.strategy:
        wl = dict(wl, strategy=a.strategy)
    model = H.HiftModel(cfg, wl["opt"], wl["m"], B, S, init_params=None, state_on_host=0 if a.state_resident else 1,
                        master_on_host=int(a.master_on_host), no_packed_copies=int(a.no_packed_copies))
    mem = model.memory()
    model.set_state_copy_engine(a.copy_engine, a.copy_blocks)
    fill_weights_on_device(model, a.seed)
    k = model.set_group_schedule(wl["strategy"], wl["m"], a.seed)
    n_total = max(a.steps + a.warmup, k)
    batches = []
    for t in range(1, n_total + 1):
        tok, lab = make_batch(wl, a.seed, t)
        batches.append((torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()))
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    # A step's cost falls linearly with the position of its group in a bottom2up or top2down sweep (61 ms with the
    # embeddings group active ... 31 ms with the head), and the metric is the mean over whole sweeps.  When the K timed
    # steps are not whole sweeps, the schedule is entered at the position that centres the part of the timed window
    # beyond its whole sweeps in the sweep: its mean position, and so its mean cost, is then the sweep's.
    # (`groups_timed` says which groups the window covered; `cycle_*` is a whole sweep timed besides.)
    # The schedule is entered by running the steps before that position, untimed, ahead of the W warm-up steps: the
    # library prefetches the state of the group its own step count says comes next.
    rem = a.steps % k
    t_first = ((k - rem) // 2 - a.warmup) % k if rem else 0
    t = 0
    loss = None

    def run(n, groups=None):
        """n scheduled steps without waiting in between; returns wall seconds."""
        nonlocal t
        model.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            t += 1
            gid = model.schedule_group_at(t)
            if groups is not None:
                groups.append(gid)
            model.step(*batches[(t - 1) % n_total], gid, want_loss=False)
        model.synchronize()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run(t_first)
    run(a.warmup)

    # timed region: K steps.  `value` is taken here, with nothing but the steps on the streams.
    h2d0, d2h0 = model.transfer_stats()
    groups_timed = []
    elapsed = run(a.steps, groups_timed)
    h2d1, d2h1 = model.transfer_stats()

    # A step's cost depends on the depth of its group, so K steps that are not whole sweeps over the k groups
    # weigh some depths more than others: one full sweep is timed as well (the timed region itself when it
    # already is whole sweeps).
    whole_sweeps = a.steps % k == 0 and a.steps > 0
    if whole_sweeps:
        cycle_s, cycle_steps = elapsed, a.steps
    else:
        run((k - t % k) % k)          # to the start of a sweep
        cycle_s, cycle_steps = run(k), k

    # Then the timed region again, over the same groups in the same order (filler steps bring the schedule back to
    # where the timed region began), with every kernel launch bracketed by HIP events on the compute stream:
    # per-class kernel time for the roofline figures (the brackets keep consecutive kernels from overlapping,
    # so this pass is a few percent slower).
    run((t_first + a.warmup - t) % k)
    model.profile_enable(True)
    groups_profiled = []
    t_prof = run(a.steps, groups_profiled)
    n_gemm, ms_gemm, fl_gemm = model.profile_read(0)
    n_att, ms_att, fl_att = model.profile_read(1)
    n_el, ms_el, by_el = model.profile_read(2)
    rowwise = model.profile_read_rowwise()
    n_opt, ms_opt, by_opt = model.profile_read(3)
    n_rest, ms_rest, fl_rest = model.profile_read(4)
    n_pack, ms_pack, by_pack = model.profile_read(5)
    model.profile_enable(False)
    # one more cycle read step by step from the library's own events on the compute stream: what a step costs
    # as a function of the group's depth (group 0 = the whole dX chain and almost no dW: the cost shape of an
    # adapter method; the top group = forward and the head only).  Reading the events waits for the streams,
    # so the state copies of consecutive steps do not overlap here as they do in the timed region.
    by_group = {}
    for _ in range(k):
        t += 1
        gid = model.schedule_group_at(t)
        model.step(*batches[(t - 1) % n_total], gid, want_loss=False)
        by_group[gid] = round(model.last_step_ms()[0], 3)
    # exposed copy time and loss of one more step
    t += 1
    loss = model.step(*batches[(t - 1) % n_total], model.schedule_group_at(t), want_loss=True)
    _step_ms, exposed = model.last_step_ms()

    tokens = a.steps * B * S
    opt_name = {"adamw": "AdamW", "adagrad": "AdaGrad"}.get(wl["opt"]["kind"], "SGD with momentum %g" % wl["opt"].get("momentum", 0.0)
                                                                if wl["opt"].get("momentum") else "SGD")
    gemm_tflops = fl_gemm / (ms_gemm * 1e-3) / 1e12 if ms_gemm > 0 else 0.0
    out = {
        "metric": "trained tokens/sec per HiFT step at 7B shape (1 GPU); MFMA util % of bf16 peak",
        "value": tokens / elapsed if elapsed > 0 else 0.0,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": 1e3 * elapsed / max(a.steps, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: LLaMA-7B-shaped decoder, 32 layers d=4096 h=32 ffn=11008 vocab=32000, "
                               f"batch {B} x seq {S}, m={wl['m']} ({k} groups), {wl['strategy']}, {opt_name}, optimizer state "
                               + ("resident in HBM" if a.state_resident else "of inactive groups in pinned host memory")
                               if a.workload == "C4" else
                               f"{a.workload}: arch {cfg['arch']}, {cfg['n_layers']} layers d={cfg['d_model']} h={cfg['n_heads']} "
                               f"ffn={cfg['d_ffn']} vocab={cfg['vocab']}" + (", tied embeddings" if cfg.get("tie_embeddings") else "")
                               + f", batch {B} x seq {S}, m={wl['m']} ({k} groups), {wl['strategy']}, {opt_name}, state "
                               + ("resident in HBM" if a.state_resident else "of inactive groups in pinned host memory"),
                   "groups": k, "tokens_per_step": B * S},
        "roofline": {
            "bound": "mfma",
            "kernel": "gemm_pk_k<128x256 tiles, bf16 out>, its fused-epilogue instantiations included: linear layers, forward and dX, "
                      "weight operand in MFMA fragment order",
            "achieved": gemm_tflops, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": gemm_tflops / BF16_PEAK_TFLOPS, "traffic": measured_traffic(),
            "traffic_source": "profiles/gemm_traffic.json: stored rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the stand-alone "
                              "kernel, weighted by one sweep's launch counts; not measured in this run; null when the "
                              "kernel source no longer matches the hash stored with them",
            "groups": groups_profiled,
            "launches": n_gemm, "avg_launch_ms": ms_gemm / max(n_gemm, 1),
            "flops_per_launch": fl_gemm / max(n_gemm, 1),
        },
        "kernel_classes_ms_per_step": {
            "linear_gemm_packed": ms_gemm / max(a.steps, 1), "linear_gemm_other": ms_rest / max(a.steps, 1),
            "attention_gemm": ms_att / max(a.steps, 1),
            "rowwise_elementwise": ms_el / max(a.steps, 1), "optimizer": ms_opt / max(a.steps, 1),
            "weight_repack": ms_pack / max(a.steps, 1),
        },
        "linear_gemm_all_tflops": (fl_gemm + fl_rest) / ((ms_gemm + ms_rest) * 1e-3) / 1e12 if ms_gemm + ms_rest > 0 else 0.0,
        "linear_gemm_other_tflops": fl_rest / (ms_rest * 1e-3) / 1e12 if ms_rest > 0 else 0.0,
        "attention_gemm_tflops": fl_att / (ms_att * 1e-3) / 1e12 if ms_att > 0 else 0.0,
        "groups_timed": groups_timed,
        "groups_timed_note": ("whole sweeps" if not rem else
                              f"{a.steps // k} whole sweep(s) + {rem} steps centred in the sweep (mean position = the sweep's): {t_first} untimed steps bring the schedule there, then the {a.warmup} warm-up steps"),
        "cycle_mean_ms": 1e3 * cycle_s / cycle_steps,
        "cycle_tokens_per_s": cycle_steps * B * S / cycle_s,
        "cycle_note": f"wall time of {cycle_steps} consecutive scheduled steps = {cycle_steps // k} whole sweep(s) over the {k} groups"
                      + (" (the timed region itself)" if whole_sweeps else " (timed after the K steps of `value`)"),
        "hbm_rooflines": hbm_rooflines(rowwise, n_opt, ms_opt, by_opt, n_pack, ms_pack, by_pack),
        "rowwise_gbps": by_el / (ms_el * 1e-3) / 1e9 if ms_el > 0 else 0.0,
        "optimizer_gbps": by_opt / (ms_opt * 1e-3) / 1e9 if ms_opt > 0 else 0.0,
        "weight_repack_gbps": by_pack / (ms_pack * 1e-3) / 1e9 if ms_pack > 0 else 0.0,
        "state_copy_gb_per_step": {"h2d": (h2d1 - h2d0) / 1e9 / max(a.steps, 1), "d2h": (d2h1 - d2h0) / 1e9 / max(a.steps, 1)},
        "exposed_state_copy_ms_last_step": exposed,
        "state_copy_engine": "copy kernel, %d workgroups" % a.copy_blocks if a.copy_engine == 1 else "hipMemcpyAsync",
        "ms_per_step_with_event_brackets": 1e3 * t_prof / max(a.steps, 1),
        "compute_stream_ms_by_group": [by_group[g] for g in sorted(by_group)],
        "last_loss": loss,
        "setup_s": setup_s,
        "memory_gb": {kk: round(mem[kk] / 1e9, 2) for kk in ("para", "gra", "sta", "pgs", "residual", "total", "pinned_total")},
        "memory_mode": {"master_on_host": bool(a.master_on_host), "packed_copies": not a.no_packed_copies},
    }
    if not a.no_cpu_baseline and a.workload in ("C4", "C5"):
        model.close()
        del model
        out["cpu_baseline"] = cpu_baseline(a.workload, a.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
