#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

One step = one pass of the whole layer over one synthetic batch already resident in HBM:
gating, micro-batch construction, the expert-block calls, the shared expert and the aggregation,
all through the C ABI.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload prefill|decode|tenants]
                    [--group-size g] [--policy p] [--shared-policy p] [--no-graph] [--no-cpu-baseline]

The timed region runs the K steps twice: once eagerly with HIP events around each grouped-GEMM
launch (these give the per-kernel durations the roofline figures use; one stream, one kernel at a
time), and once as replays of a HIP graph of the same step (no host launch cost between kernels;
the shared expert runs on a second stream inside the graph unless --overlap-shared 0).  `value` comes from the graph
replays unless --no-graph is given; both step times are in the JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak


def layer_flops_per_token(s) -> int:
    routed = 2 * 3 * s.H * s.I * s.K
    shared = 2 * 3 * s.H * s.Is
    router = 2 * s.H * s.E
    gate = 2 * s.H if s.Is > 0 else 0
    return routed + shared + router + gate


def measured_traffic(args, kernel: str, build_id: str):
    """HBM bytes per launch of `kernel` from stored rocprofv3 counter runs (FETCH_SIZE and WRITE_SIZE, each
    scaled by the same counter's reading for a plain copy of known size), or None when there is no
    such record for this workload and launch configuration, or the record was taken on another build
    of the library than the one loaded (its id is the hash of the sources it was built from)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    if args.policy != 0 or args.shared_policy != 0 or args.group_size != 0 or args.tokens != 0 or not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("build_id") != build_id:
        return None
    e = rec.get("entries", {}).get(f"{args.workload}:{kernel}")
    return None if e is None else e["hbm_bytes_per_launch"]


def mfma_sustained(moe, x, W, launches: int = 20, iters: int = 2000):
    """What the matrix pipes sustain with nothing else running (operands in registers, no memory traffic), on
    zeros and on operand values taken from the workload (token rows against weight rows): rate from HIP events
    around `launches` back-to-back launches on every compute unit, shader clock from the kernel's own counters.
    The chip lowers its clock under dense MFMA work on operands with realistic bit activity, so the second
    figure, not the published peak, is what a perfect kernel could reach on this data."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    half = 16384 // 2     # bf16 values in each half of the operand buffer
    ops = {"zeros": torch.zeros(2 * half, dtype=torch.bfloat16, device="cuda"),
           "workload_values": torch.cat([x.reshape(-1)[:half], W.reshape(-1)[:half]]).contiguous()}
    clocks = torch.zeros(2 * cus, dtype=torch.int64, device="cuda")
    out = {}
    for name, o in ops.items():
        for _ in range(3):
            moe.moe_probe_mfma(o, iters, cus, clocks)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(launches):
            moe.moe_probe_mfma(o, iters, cus, clocks)
        b.record()
        torch.cuda.synchronize()
        sec = a.elapsed_time(b) * 1e-3 / launches
        c = clocks.cpu().numpy().reshape(cus, 2).astype(float)
        flops = 2.0 * 32 * 32 * 16 * 16 * iters * 4 * cus
        out[name] = {"tflops": flops / sec / 1e12, "frac_of_peak": flops / sec / 1e12 / PEAK_MFMA_BF16_TFLOPS,
                     "shader_clock_mhz": float((c[:, 0] / (c[:, 1] / 100.0)).mean()),
                     "shader_clocks_per_mfma": float(c[:, 0].mean() / (16.0 * iters))}
    out["kernel"] = f"{cus} workgroups x 4 waves x {iters} x 16 independent v_mfma_f32_32x32x16_bf16, {launches} launches"
    return out


def run_residency(args, moe) -> int:
    """On-demand expert residency (Sec. 3: blocks are instantiated on demand and released when idle).
    Six tenants (Sec. 4.2) send decode batches of 32 tokens in turn; a strong per-tenant router bias
    keeps each tenant on its own expert subset (Sec. 3).  The routed experts' weights live in pinned
    host memory, the device holds --residency-slots blocks of --group-size experts; a step is gating,
    micro-batch construction, the read-back of the rows per expert (the orchestrator decides which
    blocks to invoke), one invocation per active block (loading it first on a miss), the shared
    expert and the aggregation."""
    n_tenants, T = 6, 32
    g_size = args.group_size if args.group_size > 0 else 6
    wl = workloads.tenants(seed=5, n_tenants=n_tenants, T_per=T)
    s = wl.shape
    res = moe.ExpertResidency(wl.Wg, wl.Wu, wl.Wd, g=g_size, slots=args.residency_slots)
    dev = {k: getattr(wl, k).cuda() for k in ("x", "Wr", "Wsg", "Wsu", "Wsd", "wgate")}
    bias = (wl.bias * args.bias_scale).cuda()
    buf = moe.LayerBuffers.allocate(T, s.H, s.E, s.K, s.I, s.Is)
    sh = (dev["Wsg"], dev["Wsu"], dev["Wsd"], dev["wgate"])
    active_blocks, active_experts = [], []

    def step(i):
        t = i % n_tenants
        x = dev["x"][t * T:(t + 1) * T]
        moe.moe_route(x, dev["Wr"], bias[t], s.K, s.renorm, buf.topk_ids, buf.topk_w)
        moe.moe_permute(buf.topk_ids, x, s.E, buf.expert_offsets, buf.src_of_row, buf.row_of_pair, None,
                        buf.workspace_permute, materialize=False)
        counts = torch.diff(buf.expert_offsets).cpu().tolist()       # synchronises: the control plane's decision
        n = res.forward_active_blocks(counts, x, buf.src_of_row, s.K, buf.expert_offsets, buf.Yp, buf.workspace,
                                      args.policy)
        moe.moe_shared_forward(x, *sh, buf.S, buf.sg, buf.workspace_shared, args.shared_policy)
        moe.moe_combine(buf.Yp, buf.row_of_pair, buf.topk_w, buf.S, buf.sg, buf.out)
        active_blocks.append(n)
        active_experts.append(sum(1 for c in counts if c > 0))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    res.hits = res.misses = 0
    res.bytes_copied = 0
    del active_blocks[:], active_experts[:]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    full = 3 * s.E * s.I * s.H * 2
    out = {
        "metric": "moe_layer_tokens_per_s", "value": T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"residency: {n_tenants} tenants in turn, {T} tokens per step, Qwen1.5-MoE-2.7B-shaped layer",
                   "T": T, "H": s.H, "E": s.E, "K": s.K, "I": s.I, "Is": s.Is, "experts_per_block": g_size,
                   "blocks": len(res.blocks), "slots": res.slots, "bias_scale": args.bias_scale, "launch": "eager"},
        "residency": {"resident_routed_weight_bytes": res.resident_bytes(), "all_routed_weight_bytes": full,
                      "resident_fraction": res.resident_bytes() / full,
                      "block_hit_rate": res.hits / max(1, res.hits + res.misses),
                      "host_to_device_bytes_per_step": res.bytes_copied / args.steps,
                      "active_blocks_per_step": float(np.mean(active_blocks)),
                      "active_experts_per_step": float(np.mean(active_experts))},
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="prefill", choices=["prefill", "decode", "tenants", "stack", "residency"])
    ap.add_argument("--residency-slots", type=int, default=4,
                    help="residency workload: expert blocks (of --group-size experts, default 6) the device pool holds")
    ap.add_argument("--bias-scale", type=float, default=4.0,
                    help="residency workload: factor on the tenants' router biases (how strongly a tenant keeps to "
                         "its own expert subset)")
    ap.add_argument("--layers", type=int, default=24, help="layers of the stack workload")
    ap.add_argument("--tokens", type=int, default=0,
                    help="batch size T of the prefill (Zipf-skewed routing) or decode (unbiased routing) workload instead of "
                         "its own 4096 / 128: for sweeps over the batch size (0: the workload's own)")
    ap.add_argument("--group-size", type=int, default=0, help="experts per expert block (0: one block)")
    ap.add_argument("--route-per-tenant", action="store_true",
                    help="tenants/stack workloads: one gating launch per tenant slice instead of one for the batch")
    ap.add_argument("--policy", type=int, default=0)
    ap.add_argument("--shared-policy", type=int, default=0)
    ap.add_argument("--block-streams", type=int, default=1,
                    help="issue the expert-block calls round-robin over this many streams (blocks are independent)")
    ap.add_argument("--fused-gather", type=int, default=1,
                    help="1 (default): no permuted copy of the tokens, the block calls read x through src_of_row; "
                         "0: moe_permute writes Xp and the block calls read it")
    ap.add_argument("--fused-shared", type=int, default=0,
                    help="1: the first block call also runs the shared experts (as Is / I experts of the routed size on "
                         "every token) in the same two launches, where the library supports it (prefill-sized "
                         "batches); 0 (default, measured faster): the shared expert is a call of its own")
    ap.add_argument("--balanced-blocks", type=int, default=0,
                    help="with --group-size g: form the E/g blocks by observed load (rows per expert of a warm-up "
                         "step, heaviest expert first to the lightest block) instead of as id ranges")
    ap.add_argument("--orchestrator", default="shared", choices=["shared", "private"],
                    help="tenants workload: 'shared' = one orchestrator batches all tenants' tokens into one "
                         "micro-batch per expert block (Sec. 3, Sec. 4.1); 'private' = one orchestrator per tenant, "
                         "each with its own gating, micro-batches, block invocations and aggregation")
    ap.add_argument("--tenant-streams", type=int, default=1,
                    help="private orchestrators: issue the tenants' layers round-robin over this many streams")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--overlap-shared", type=int, default=-1,
                    help="1: shared expert on a second stream, concurrent with the routed path; 0: one stream; "
                         "-1 (default): on (the shared expert depends on x only, so it fills the gaps "
                         "the routing, permute and tail phases of the routed path leave)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the timed steps, run three plain device copies of this many MiB (a kernel of "
                         "known HBM traffic, to scale profiler byte counters taken in the same run)")
    ap.add_argument("--with-decode", type=int, default=1,
                    help="prefill workload: 1 (default) also measures the decode batch (T = 128) in the same run and "
                         "attaches it to the JSON line under \"decode\"; 0: prefill only")
    ap.add_argument("--mfma-probe", type=int, default=1,
                    help="1: also report what the matrix pipes sustain on zeros and on the workload's values with nothing "
                         "else running (prefill-sized workloads; adds about 30 ms of GPU time)")
    ap.add_argument("--tile-clocks", type=int, default=1,
                    help="1: the MFMA tile kernels of the eager region record their workgroups' clocks (shader clock held, "
                         "share of the K loops); reported per kernel under kernels.*.tile_clocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU; the layer forward has no multi-GPU path "
              "(token batches would shard without any exchange). Run with --gpus 1.", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        return 3

    import paper_2604_26881_amd as moe
    moe.load()

    if args.workload == "residency":
        return run_residency(args, moe)

    out = run_layer_workload(args, moe, cpu_baseline=not args.no_cpu_baseline)
    if out is None:
        return 2
    if args.workload == "prefill" and args.with_decode:
        # the weight-streaming regime in the same run: the decode batch (T = 128) through the same calls,
        # measured the same way, its own roof (HBM) attached beside the prefill figures
        dargs = argparse.Namespace(**vars(args))
        dargs.workload = "decode"
        dargs.steps, dargs.warmup = max(args.steps, 50), max(args.warmup, 10)
        d = run_layer_workload(dargs, moe, cpu_baseline=False)
        out["decode"] = {k: d[k] for k in ("value", "unit", "ms_per_step", "ms_per_step_eager", "ms_per_step_graph",
                                           "steps", "warmup", "config", "layer_gbs", "layer_frac_of_hbm_peak",
                                           "layer_bytes_algorithmic", "roofline", "kernels")}
    print(json.dumps(out))
    return 0


def run_layer_workload(args, moe, cpu_baseline: bool):
    """Measures one workload (prefill, decode, tenants or stack) and returns the record of its JSON line."""
    stack = args.workload == "stack"
    if stack:
        # 24 Qwen-shaped MoE layers (no attention), independent weights per layer drawn on the GPU
        # (seed 1000 + layer), T = 2048 tokens, residual add + RMS normalisation between layers
        s = workloads.Shape(T=2048, **workloads.QWEN)
        wl = workloads.Workload(name="stack", shape=s, x=workloads.tokens(s.T, s.H, 4242, torch.bfloat16),
                                **workloads.stack_layer_weights(0, device="cuda"))
        layer_w = [wl.tensors()] + [workloads.stack_layer_weights(l, device="cuda") for l in range(1, args.layers)]
        g = wl.to("cuda")
    else:
        make = {"prefill": workloads.prefill, "decode": workloads.decode, "tenants": workloads.tenants}[args.workload]
        if args.tokens > 0 and args.workload == "tenants":
            print("bench.py: --tokens applies to the prefill and decode workloads", file=sys.stderr)
            return None
        wl = make(T=args.tokens) if args.tokens > 0 else make()
        s = wl.shape
        g = wl.to("cuda")
        layer_w = [g.tensors()]
    n_layers = len(layer_w)
    shared = (g.Wsg, g.Wsu, g.Wsd, g.wgate) if s.Is > 0 else None
    x_stack = torch.empty_like(g.x) if stack else None
    groups = workloads.partition(s.E, args.group_size) if args.group_size > 0 else [(0, s.E)]
    buf = moe.LayerBuffers.allocate(s.T, s.H, s.E, s.K, s.I, s.Is)

    seg = moe.segment_offsets(wl.tenant_rows, s.T, "cuda") if wl.tenant_rows is not None else None

    def route(x, w):
        if seg is not None and not args.route_per_tenant:   # one gating launch, one bias row per tenant slice
            moe.moe_route_segments(x, w["Wr"], w["bias"], seg, s.K, s.renorm, buf.topk_ids, buf.topk_w)
        elif wl.tenant_rows is not None:
            for i, (a, b) in enumerate(wl.tenant_rows):
                moe.moe_route(x[a:b], w["Wr"], w["bias"][i], s.K, s.renorm, buf.topk_ids[a:b], buf.topk_w[a:b])
        else:
            moe.moe_route(x, w["Wr"], w.get("bias"), s.K, s.renorm, buf.topk_ids, buf.topk_w)

    # phase bits of the *_ex policy word: 0x100 = gate/up kernel only, 0x200 = down kernel only
    GU, DN = 0x100, 0x200
    names = ["routed_gateup", "routed_down", "shared_gateup", "shared_down"]
    overlap = True if args.overlap_shared < 0 else bool(args.overlap_shared)
    overlap = overlap and shared is not None
    side_stream = torch.cuda.Stream() if overlap else None
    block_streams = [torch.cuda.Stream() for _ in range(args.block_streams)] if args.block_streams > 1 else []

    fused = bool(args.fused_gather)
    # the shared experts inside the first block call (needs the gather form and id-range blocks)
    fshared = bool(args.fused_shared and fused and shared is not None and buf.S_parts is not None
                   and not args.balanced_blocks and args.block_streams <= 1)
    if fshared:
        names = ["fused_gateup", "fused_down"]
        overlap, side_stream = False, None

    block_lists = None     # per block an int32 device tensor of expert ids (load-balanced blocks)

    def block_call(x, w, lo, hi, policy):
        if fshared and lo == groups[0][0]:
            moe.moe_expert_group_forward_fused(lo, hi, x, buf.src_of_row, s.K, buf.expert_offsets, w["Wg"], w["Wu"],
                                               w["Wd"], w["Wsg"], w["Wsu"], w["Wsd"], w["wgate"], buf.Yp, buf.S_parts,
                                               buf.sg, buf.workspace_fused, policy)
            return
        if block_lists is not None:
            moe.moe_expert_list_forward(block_lists[lo], x if fused else buf.Xp, buf.src_of_row if fused else None, s.K,
                                        buf.expert_offsets, w["Wg"], w["Wu"], w["Wd"], buf.Yp, buf.workspace, policy)
            return
        if fused:
            moe.moe_expert_group_forward_gather(lo, hi, x, buf.src_of_row, s.K, buf.expert_offsets, w["Wg"], w["Wu"],
                                                w["Wd"], buf.Yp, buf.workspace, policy)
        else:
            moe.moe_expert_group_forward(lo, hi, buf.Xp, buf.expert_offsets, w["Wg"], w["Wu"], w["Wd"], buf.Yp,
                                         buf.workspace, policy)

    def run_blocks(x, w, policy):
        """One block invocation per expert block; with several streams the independent blocks overlap."""
        if not block_streams:
            for lo, hi in groups:
                block_call(x, w, lo, hi, policy)
            return
        main = torch.cuda.current_stream()
        for st in block_streams:
            st.wait_stream(main)
        for i, (lo, hi) in enumerate(groups):
            with torch.cuda.stream(block_streams[i % len(block_streams)]):
                block_call(x, w, lo, hi, policy)
        for st in block_streams:
            main.wait_stream(st)

    # clock records of the four grouped-GEMM launches (one buffer each, room for 1024 workgroups)
    clock_bufs = ([torch.zeros(4 * 1024, dtype=torch.int64, device="cuda") for _ in range(4)]
                  if args.tile_clocks and len(groups) == 1 and not fshared else [])

    def layer_step(x, w, events=None):
        sh = (w["Wsg"], w["Wsu"], w["Wsd"], w["wgate"]) if s.Is > 0 else None
        if overlap and events is None:
            # the shared expert depends on x only: it forks off here to the second stream.  The routed
            # path is enqueued first and stays on the stream that also runs the aggregation, so that
            # the step's critical path (gating -> ... -> aggregation) never waits for a signal from
            # another hardware queue (measured: about 10 us each at the fork and at the join); the
            # short side branch pays them instead
            fork = torch.cuda.Event()
            fork.record()
        route(x, w)
        moe.moe_permute(buf.topk_ids, x, s.E, buf.expert_offsets, buf.src_of_row, buf.row_of_pair, buf.Xp,
                        buf.workspace_permute, materialize=not fused)
        if fshared:
            if events is None:
                run_blocks(x, w, args.policy)
            else:
                ev = [[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in names]
                for i, phase in enumerate((GU, DN)):
                    ev[i][0].record()
                    run_blocks(x, w, args.policy | phase)
                    ev[i][1].record()
                events.append(ev)
            moe.moe_combine_parts(buf.Yp, buf.row_of_pair, buf.topk_w, buf.S_parts, buf.sg, buf.out)
            return
        if events is None:
            run_blocks(x, w, args.policy)
            if sh is not None and not overlap:
                moe.moe_shared_forward(x, *sh, buf.S, buf.sg, buf.workspace_shared, args.shared_policy)
            if overlap:
                side_stream.wait_event(fork)
                with torch.cuda.stream(side_stream):
                    # 0x400: the shared expert's first kernel leaves room on the CUs for the gating and
                    # permute kernels that run at the same time on the main stream
                    moe.moe_shared_forward(x, *sh, buf.S, buf.sg, buf.workspace_shared, args.shared_policy | 0x400)
                torch.cuda.current_stream().wait_stream(side_stream)
        else:
            # same kernels, launched one per call so that events can bracket each of them
            # (each launch also records its workgroups' clocks into a buffer of its own when the MFMA tile kernels
            # serve it; the last step's records are read after the region)
            ev = [[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in names]
            clk = (lambda i: moe.moe_tile_clock_buffer(clock_bufs[i])) if clock_bufs else (lambda i: None)
            clk(0)
            ev[0][0].record()
            run_blocks(x, w, args.policy | GU)
            ev[0][1].record()
            clk(1)
            ev[1][0].record()
            run_blocks(x, w, args.policy | DN)
            ev[1][1].record()
            if sh is not None:
                clk(2)
                ev[2][0].record()
                # (with the same "leave room" bit as in the timed step, so the figure is for the shape the step runs)
                moe.moe_shared_forward(x, *sh, buf.S, buf.sg, buf.workspace_shared,
                                       args.shared_policy | GU | (0x400 if overlap else 0))
                ev[2][1].record()
                clk(3)
                ev[3][0].record()
                moe.moe_shared_forward(x, *sh, buf.S, buf.sg, buf.workspace_shared, args.shared_policy | DN)
                ev[3][1].record()
            if clock_bufs:
                moe.moe_tile_clock_buffer(None)
            events.append(ev)
        moe.moe_combine(buf.Yp, buf.row_of_pair, buf.topk_w, buf.S, buf.sg, buf.out)

    private = args.orchestrator == "private"
    if private and wl.tenant_rows is None:
        print("bench.py: --orchestrator private needs the tenants workload", file=sys.stderr)
        return None
    if private:
        tbufs = [moe.LayerBuffers.allocate(b - a, s.H, s.E, s.K, s.I, s.Is) for a, b in wl.tenant_rows]
        tstreams = [torch.cuda.Stream() for _ in range(args.tenant_streams)] if args.tenant_streams > 1 else []

    def tenant_layer(i, a, b):
        w = layer_w[0]
        moe.moe_layer_forward(g.x[a:b], w["Wr"], w["bias"][i:i + 1], w["Wg"], w["Wu"], w["Wd"], shared, s.K, s.renorm,
                              groups=groups, buf=tbufs[i], tenant_rows=[(0, b - a)], policy=args.policy,
                              shared_policy=args.shared_policy, fused_gather=fused)

    def step_private():
        """Every tenant's tokens go through their own gating, micro-batching, block calls and aggregation."""
        if not tstreams:
            for i, (a, b) in enumerate(wl.tenant_rows):
                tenant_layer(i, a, b)
            return
        main = torch.cuda.current_stream()
        for st in tstreams:
            st.wait_stream(main)
        for i, (a, b) in enumerate(wl.tenant_rows):
            with torch.cuda.stream(tstreams[i % len(tstreams)]):
                tenant_layer(i, a, b)
        for st in tstreams:
            main.wait_stream(st)

    def step(events=None):
        if private and events is None:
            return step_private()
        x = g.x
        for w in layer_w:
            layer_step(x, w, events)
            if stack:                      # residual add + RMS normalisation feeds the next layer
                moe.moe_residual_norm(x, buf.out, x_stack)
                x = x_stack

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.balanced_blocks and len(groups) > 1 and not stack:
        # the load observed in the warm-up steps decides the blocks of the timed steps (same batch here)
        observed = torch.diff(buf.expert_offsets).cpu().tolist()
        lists = moe.balanced_blocks(observed, len(groups))
        block_lists = [torch.tensor(b, dtype=torch.int32, device="cuda") for b in lists]
        block_rows = [sum(observed[e] for e in b) for b in lists]
        range_rows = [sum(observed[lo:hi]) for lo, hi in groups]
        groups = [(i, i + 1) for i in range(len(lists))]     # block_call indexes block_lists by lo
        for _ in range(2):
            step()
        torch.cuda.synchronize()
    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region 1: eager, events around the four grouped-GEMM launches
    events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    if private:   # the per-kernel events above are those of the shared orchestrator; time the private step itself
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kern_ms = {}
    for i, n in enumerate(names):
        if shared is None and i >= 2:
            continue
        kern_ms[n] = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for ev in events]))   # per layer

    # ---- timed region 2: the same step as HIP-graph replays
    graph_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(max(3, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    ms = graph_ms if graph_ms is not None else eager_ms
    tokens_per_s = s.T / (ms * 1e-3)
    flop_tok = layer_flops_per_token(s)
    flop_tok *= n_layers
    layer_tflops = flop_tok * s.T / (ms * 1e-3) / 1e12

    # ---- roofline of the dominant grouped-GEMM kernel
    counts = torch.diff(buf.expert_offsets).cpu().numpy()
    active = int((counts > 0).sum())
    P = s.P
    alg_flops = {"routed_gateup": 2 * 2 * P * s.H * s.I, "routed_down": 2 * P * s.H * s.I,
                 "shared_gateup": 2 * 2 * s.T * s.H * s.Is, "shared_down": 2 * s.T * s.H * s.Is}
    alg_bytes = {"routed_gateup": active * 2 * s.I * s.H * 2 + P * s.H * 2 + P * s.I * 2,
                 "routed_down": active * s.I * s.H * 2 + P * s.I * 2 + P * s.H * 2,
                 "shared_gateup": 2 * s.Is * s.H * 2 + s.T * s.H * 2 + s.T * s.Is * 2,
                 "shared_down": s.Is * s.H * 2 + s.T * s.Is * 2 + s.T * s.H * 2}
    if fshared:
        # routed and shared experts in the same launches; the shared experts' outputs are written as
        # Is / I tensors [T,H] (one per shared expert) instead of one
        n_sets = int(buf.S_parts.shape[0])
        alg_flops = {"fused_gateup": alg_flops["routed_gateup"] + alg_flops["shared_gateup"],
                     "fused_down": alg_flops["routed_down"] + alg_flops["shared_down"]}
        alg_bytes = {"fused_gateup": alg_bytes["routed_gateup"] + alg_bytes["shared_gateup"],
                     "fused_down": alg_bytes["routed_down"] + alg_bytes["shared_down"] + (n_sets - 1) * s.T * s.H * 2}
    dom = max(kern_ms, key=kern_ms.get)
    launches = 1 if dom.startswith("shared") else len(groups)
    dur_s = kern_ms[dom] * 1e-3 / launches      # average duration of one launch
    # Which roof: the grouped GEMMs of prefill-sized batches are matrix-core work (the target is a
    # fraction of the bf16 MFMA peak); at decode sizes the same kernels stream weights (HBM).
    # Both figures of every kernel are in "kernels".
    # (the library's own switch to the weight-streaming kernels, or the caller's choice of them)
    streaming = (args.policy & 0xff) == 9 or ((args.policy & 0xff) == 0 and s.E >= 16 and P // s.E <= 26)
    if streaming:
        achieved = alg_bytes[dom] / launches / dur_s / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    else:
        achieved = alg_flops[dom] / launches / dur_s / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_MFMA_BF16_TFLOPS, "traffic": None}
    roof["traffic"] = measured_traffic(args, dom, moe.build_id())
    sustained = None
    if args.mfma_probe and not streaming:
        sustained = mfma_sustained(moe, g.x, g.Wg)
        roof["frac_of_sustained_on_workload_values"] = achieved / sustained["workload_values"]["tflops"]
    roof.update({"kernel": dom, "launch_us": dur_s * 1e6, "launches_per_step": launches,
                 "algorithmic_flops_per_launch": alg_flops[dom] / launches,
                 "algorithmic_bytes_per_launch": alg_bytes[dom] / launches})
    kernels = {n: {"ms_per_step": kern_ms[n], "tflops": alg_flops[n] / (kern_ms[n] * 1e-3) / 1e12,
                   "gbs": alg_bytes[n] / (kern_ms[n] * 1e-3) / 1e9} for n in kern_ms}
    # the shader clock the chip held inside the tile kernels of the last eager step (workgroups that recorded)
    for i, n in enumerate(names):
        if clock_bufs and n in kernels:
            c = clock_bufs[i].cpu().numpy().reshape(-1, 4).astype(float)
            c = c[c[:, 3] > 0]
            if len(c):
                kernels[n]["tile_clocks"] = {
                    "workgroups": int(len(c)), "tiles": int(c[:, 3].sum()),
                    "shader_clock_mhz": float((c[:, 0] / (c[:, 1] / 100.0)).mean()),
                    "k_loop_share_of_workgroup_clocks": float(c[:, 2].sum() / c[:, 0].sum()),
                    "k_loop_shader_clocks_per_tile": float(c[:, 2].sum() / c[:, 3].sum()),
                    # a persistent workgroup's lifetime (100 MHz ticks): they start together, so the spread is the
                    # launch's tail (compute units idle while the last workgroups finish)
                    "workgroup_lifetime_us": {"min": float(c[:, 1].min() / 100.0), "mean": float(c[:, 1].mean() / 100.0),
                                              "max": float(c[:, 1].max() / 100.0)}}

    # whole-layer fractions against both roofs (weights of active experts + shared + activations)
    layer_bytes = (sum(alg_bytes[n] for n in kern_ms) + s.E * s.H * 2 + 2 * s.T * s.H * 2 + 2 * P * s.H * 2) * n_layers
    out = {
        "metric": "moe_layer_tokens_per_s", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": (f"stack: {n_layers} Qwen1.5-MoE-2.7B-shaped MoE layers, T={s.T}" if stack else
                                f"{args.workload}: Qwen1.5-MoE-2.7B-shaped layer, T={s.T}"), "layers": n_layers,
                   "T": s.T, "H": s.H,
                   "E": s.E, "K": s.K, "I": s.I, "Is": s.Is, "renorm": s.renorm, "expert_blocks": len(groups),
                   "policy": args.policy, "shared_policy": args.shared_policy,
                   "launch": "hip graph replay" if graph_ms is not None else "eager",
                   "block_streams": max(1, args.block_streams),
                   "blocks": ({"formed": "by observed load", "rows_per_block": block_rows, "rows_per_range_block": range_rows}
                              if block_lists is not None else "id ranges"),
                   "orchestrator": (f"private: {len(wl.tenant_rows)} tenants, each its own layer pass over "
                                    f"{max(1, args.tenant_streams)} stream(s); per-kernel figures are the shared orchestrator's"
                                    if private else "shared"),
                   "token_gather": "inside the gate/up kernel (no permuted copy)" if fused else "permuted copy Xp",
                   "shared_expert": ("inside the first block call, as Is / I experts on every token" if fshared else
                                     "second stream, concurrent with the routed path" if overlap else "same stream"),
                   "active_experts": active, "rows_per_expert_max": int(counts.max()),
                   "rows_per_expert_median": float(np.median(counts)),
                   "rows_per_expert_histogram": {
                       "bin_upper_edges": [0, 32, 64, 128, 160, 256, 320, 512, 1024, "inf"],
                       "experts": [int(v) for v in np.histogram(
                           counts, bins=[-0.5, 0.5, 32.5, 64.5, 128.5, 160.5, 256.5, 320.5, 512.5, 1024.5, 1e9])[0]]}},
        "ms_per_step_eager": eager_ms, "ms_per_step_graph": graph_ms,
        "layer_tflops": layer_tflops, "layer_frac_of_mfma_peak": layer_tflops / PEAK_MFMA_BF16_TFLOPS,
        "layer_gbs": layer_bytes / (ms * 1e-3) / 1e9, "layer_frac_of_hbm_peak": layer_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "flop_per_token": flop_tok, "layer_bytes_algorithmic": layer_bytes, "roofline": roof, "kernels": kernels, "build_id": moe.build_id(),
    }
    if sustained is not None:
        out["mfma_sustained"] = sustained

    # ---- CPU baseline: the oracle, per-token definition, on a bounded sample of the same batch
    if cpu_baseline:
        import oracle
        orc = oracle.Oracle("f64")
        d = wl.f32_numpy()
        cores = orc.num_threads()
        sh = None if s.Is == 0 else (d["Wsg"], d["Wsu"], d["Wsd"], d["wgate"])
        done, t_cpu, batch = 0, 0.0, max(cores * 4, 16)
        while t_cpu < args.cpu_seconds and done < s.T:
            tok = np.arange(done, min(s.T, done + batch), dtype=np.int32)
            bias = d["bias"]
            if wl.tenant_rows is not None:
                bias = bias[0]
            t0 = time.perf_counter()
            orc.token_forward(tok, d["x"], d["Wr"], bias, d["Wg"], d["Wu"], d["Wd"], sh, s.K, s.renorm)
            t_cpu += time.perf_counter() - t0
            done += len(tok)
        out["cpu_baseline"] = {"value": done / t_cpu, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {done} tokens of the same batch, float64 per-token definition "
                                         f"(the checker as it stands: gcc -O2, no fast-math, OpenMP over tokens), "
                                         f"{t_cpu:.1f} s"}
        if stack:   # one layer was timed; the stack repeats it n_layers times per token
            out["cpu_baseline"]["value"] /= n_layers
            out["cpu_baseline"]["sample"] += f"; layer 0 only, divided by {n_layers} layers"
    return out


if __name__ == "__main__":
    sys.exit(main())
