"""Benchmark of the hybrid-attention forward on one MI355X.

One step = one forward of the whole hot path (softmax-key compaction, state pass, fused query
kernel) over one batch of synthetic input that is already resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # 256 CU x 2.4 GHz x 4096 flop/clk/CU, dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def cpu_baseline(w, heads=12):
    """fp64 oracle on the host cores for a bounded sample of the same workload: the full forward
    (every key, every query row) of `heads` of the B*H (batch, head) pairs, scaled linearly to all of
    them (heads are independent problems of identical cost)."""
    from oracle import hybrid_attn_oracle as O
    from paper_2509_24899_amd import workloads as W
    heads = min(heads, w.H)
    inp = W.make_inputs(W.replace(w, B=1), heads=heads)
    fq = O.FeatureMap(inp.phi_q.w1, inp.phi_q.b1, inp.phi_q.w2, inp.phi_q.b2, w.poly_degree)
    fk = O.FeatureMap(inp.phi_k.w1, inp.phi_k.b1, inp.phi_k.w2, inp.phi_k.b2, w.poly_degree)
    t0 = time.perf_counter()
    split = O.BlockSplit(w.R, w.split_granularity) if w.split_granularity > 1 else w.R
    if w.local_window > 0:
        O.hybrid_attn_local_window(inp.q, inp.k, inp.v, fq, fk, w.scale, 2 * w.block_size, w.local_window // (2 * w.block_size))
    elif 0 < w.causal_chunk < w.N:
        O.hybrid_attn_chunk_causal(inp.q, inp.k, inp.v, fq, fk, split, w.scale, w.causal_chunk)
    else:
        O.hybrid_attn(inp.q, inp.k, inp.v, fq, fk, split, w.scale)
    t_sample = time.perf_counter() - t0
    t_full = t_sample * (w.B * w.H) / heads
    return {"value": w.B * w.N / t_full, "unit": "tokens/s", "cores": host_threads(), "cpu_model": cpu_model(), "kind": "oracle",
            "sample": f"full fp64 oracle forward (all {w.N} rows, all keys) of {heads} of the {w.B * w.H} (batch, head) "
                      f"pairs: {t_sample:.1f} s, scaled to all pairs: {t_full:.1f} s per forward"}


def rate_selection_mode(args, w, ha, W, torch, q, k, v, fq, fk, out):
    """Sec. 3.3 on measured costs: c_R = time of one layer of this shape at rate R (equal for all layers,
    the shape being equal), e_{l,R} synthetic (the real ones come out of distillation, which needs the
    model's weights): e_{l,1} = 0 and e_{l,R} = a_l (1 - 1/R)^2 with a_l log-normal, seed 0."""
    import numpy as np
    rates, n_layers = (1, 2, 4, 8), 30
    dev = q.device

    def run_layer(R, ws):
        ha.hybrid_attn_forward(q, k, v, None if R == 1 else fq, None if R == 1 else fk, R, w.block_size, w.scale,
                               out=out, workspace=ws)

    ws_bytes = max(ha.hybrid_attn_workspace_bytes(ha.make_problem(q, R, w.block_size, w.scale),
                                                  None if R == 1 else fq, None if R == 1 else fk) for R in rates)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    cost_ms = []
    for R in rates:
        for _ in range(2):
            run_layer(R, ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            run_layer(R, ws)
        e1.record()
        torch.cuda.synchronize()
        cost_ms.append(e0.elapsed_time(e1) / args.steps)
    if args.measured_errors:
        # e_{l,R} = || y - y_hat ||_1 / numel with the teacher output cached once (the inputs are shared) and
        # layer l's own feature maps (untrained, seed 1000 + l): the pipeline of Alg. 1's loss line, not its values
        s_ = w.d ** -0.5
        dt = q.dtype
        y_t = torch.empty_like(q)
        y_s = torch.empty_like(q)
        ha.hybrid_attn_forward(q, k, v, None, None, 1, w.block_size, w.scale, out=y_t, workspace=ws)
        ws_vd = None
        err, loss_ms = [], []
        for l in range(n_layers):
            g = torch.Generator(device=dev).manual_seed(1000 + l)
            maps = [ha.FeatureMap((torch.randn(w.H, w.d_hidden, w.d, generator=g, device=dev) * s_).to(dt),
                                  torch.randn(w.H, w.d_hidden, generator=g, device=dev) * 0.1,
                                  (torch.randn(w.H, w.d_feat, w.d_hidden, generator=g, device=dev) * w.d_hidden ** -0.5).to(dt),
                                  torch.randn(w.H, w.d_feat, generator=g, device=dev) * 0.1, w.poly_degree) for _ in range(2)]
            row = [0.0]
            for R in rates[1:]:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                loss, _, _ = ha.hybrid_attn_value_distill_loss(q, k, v, maps[0], maps[1], R, w.block_size, w.scale,
                                                               y_teacher=y_t, teacher_is_cached=True, y_student=y_s)
                e1.record()
                torch.cuda.synchronize()
                row.append(float(loss[0].item()) / q.numel())
                loss_ms.append(e0.elapsed_time(e1))
            err.append(row)
    else:
        rng = np.random.default_rng(0)
        a = rng.lognormal(0.0, 1.0, size=n_layers)
        err = [[float(a[l] * (1.0 - 1.0 / R) ** 2) for R in rates] for l in range(n_layers)]
    cost = [list(cost_ms) for _ in range(n_layers)]
    budget = args.select_rates * n_layers * cost_ms[0]
    t0 = time.perf_counter()
    sel = ha.hybrid_attn_select_rates(cost, err, budget)
    solve_ms = (time.perf_counter() - t0) * 1e3
    rec = {"metric": "hybrid-attention 30-layer stack with selected block rates", "unit": "ms", "n_gpus": 1,
           "higher_is_better": False, "data": "synthetic", "dtype": "bf16",
           "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d_head": w.d, "layers": n_layers,
                      "candidate_rates": list(rates), "beta": args.select_rates},
           "layer_cost_ms": dict(zip(map(str, rates), cost_ms)), "budget_ms": budget, "solve_ms": solve_ms,
           "errors": "value-distillation loss per element, untrained per-layer feature maps" if args.measured_errors
                     else "synthetic: a_l (1 - 1/R)^2, a_l log-normal, seed 0"}
    if args.measured_errors:
        rec["loss_eval_ms_mean"] = sum(loss_ms) / len(loss_ms)
    if sel is None:
        rec.update({"value": None, "note": "no assignment fits the budget"})
        print(json.dumps(rec), flush=True)
        return
    choice, total_cost, total_err = sel
    layer_rates = [rates[c] for c in choice]
    for R in layer_rates[:3]:
        run_layer(R, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for R in layer_rates:
        run_layer(R, ws)
    e1.record()
    torch.cuda.synchronize()
    homog = {str(R): {"cost_ms": n_layers * cost_ms[i], "error": sum(e[i] for e in err)} for i, R in enumerate(rates)}
    rec.update({"value": e0.elapsed_time(e1), "predicted_ms": total_cost, "selected_rates": layer_rates,
                "selected_error": total_err, "homogeneous": homog,
                "rate_histogram": {str(R): layer_rates.count(R) for R in rates}})
    print(json.dumps(rec), flush=True)


def distill_step_mode(args, w, ha, torch, q, k, v, fq, fk):
    """One student update of the attention-distillation loop (Sec. 3.3, Alg. 1, inner loop) on the cached teacher
    output: student forward, loss, gradient with respect to phi_q and phi_k.  Prints one JSON line."""
    assert w.R != 1, "the gradient needs linear tokens"
    prob = ha.make_problem(q, w.rate, w.block_size, w.scale)
    lib_ws = torch.empty(max(ha.hybrid_attn_value_distill_grad_workspace_bytes(prob, fq, fk), 256), dtype=torch.uint8,
                         device=q.device)
    loss, gq, gk, yt, ys, rd = ha.hybrid_attn_value_distill_grad(q, k, v, fq, fk, w.rate, w.block_size, w.scale, workspace=lib_ws)
    torch.cuda.synchronize()

    # the update line of Alg. 1 with the optimiser of the paper's training details (AdamW, 1e-3): fp32 master copies of
    # the weights, the forward reads their io-dtype copies; the biases are fp32 already
    names = [n for n in ("w1", "b1", "w2", "b2", "w_mid", "b_mid") if getattr(fq, n, None) is not None]
    state = []
    for fm, g in ((fq, gq), (fk, gk)):
        for n in names:
            t = getattr(fm, n)
            master = t if t.dtype == torch.float32 else t.float()
            state.append(dict(master=master, io=None if master is t else t, grad=g[n], m=torch.zeros_like(master),
                              v=torch.zeros_like(master)))
    step_no = [0]

    def full_step():
        # the gradient call writes into fresh tensors; the timed loop keeps the first call's as the update's input,
        # which changes no cost: the update reads a gradient of the same size
        ha.hybrid_attn_value_distill_grad(q, k, v, fq, fk, w.rate, w.block_size, w.scale, y_teacher=yt, teacher_is_cached=True,
                                          y_student=ys, row_den=rd, workspace=lib_ws)
        step_no[0] += 1
        for s in state:
            ha.hybrid_attn_param_update(s["master"], s["grad"], 1e-3, kind=ha.HA_OPT_ADAMW, m=s["m"], v=s["v"], step=step_no[0],
                                        grad_scale=1.0 / (w.B * w.N * w.d), param_io=s["io"])

    def backward_only():
        ha.hybrid_attn_value_distill_grad(q, k, v, fq, fk, w.rate, w.block_size, w.scale, y_teacher=yt, teacher_is_cached=True,
                                          y_student=ys, row_den=rd, student_is_cached=True, workspace=lib_ws)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps, e0.elapsed_time(e1) / args.steps

    settle_clocks(torch, full_step)           # (defined below; the GPU leaves its idle clock state)
    wall_full, ev_full = timed(full_step)
    _, ev_bwd = timed(backward_only)          # state pass + loss + backward (no student query kernel)
    n_l = w.n_linear
    # algorithmic flops of the backward pass per token: map recomputed (d Hd + Hd F), dphi (F d), W2^T du (F Hd),
    # dW2 (F Hd), dW1 (Hd d); queries also dS (F d); a middle layer adds its forward, its transpose and its weight
    # gradient (3 Dm Hd) and makes Dm the last layer's input width; 2 flops per multiply-add
    kl = w.d_mid if w.d_mid else w.d_hidden
    per_q = 2.0 * (w.d * w.d_hidden + 3 * w.d_mid * w.d_hidden + kl * w.d_feat + w.d_feat * w.d + 2 * w.d_feat * kl + w.d_hidden * w.d + w.d_feat * w.d)
    per_k = per_q - 2.0 * w.d_feat * w.d
    bwd_flops = w.B * w.H * (w.N * per_q + n_l * per_k)
    rec = {
        "metric": "value-distillation step tokens/s", "value": w.B * w.N / (wall_full * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_full, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d_head": w.d, "io_dtype": w.dtype, "hybrid_rate_R": w.R,
                   "block_size": w.block_size, "feature_map": f"{w.d}->{w.d_hidden}->" + (f"{w.d_mid}->" if w.d_mid else "") + f"{w.d_feat}, P={w.poly_degree}",
                   "step": "student forward + loss + gradient of phi_q, phi_k + AdamW update (teacher output cached)"},
        "step_ms_events": ev_full, "backward_with_state_pass_and_loss_ms": ev_bwd,
        "roofline": {"bound": "mfma", "kernel": ("grad_kernel (query pass + key pass) with its small helpers" if w.d_hidden == w.d and w.d_feat == w.d
                                                    else "the pass-per-step backward of wider maps, all kernels"), "achieved":
                     bwd_flops / (ev_bwd * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": bwd_flops / (ev_bwd * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "kernel_ms": ev_bwd, "traffic": None},
        "loss": float(loss[0].item()),
        "grad_norms": {side + "." + n: float(g[n].double().norm().item()) for side, g in (("phi_q", gq), ("phi_k", gk)) for n in g},
    }
    print(json.dumps(rec), flush=True)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        return os.cpu_count() or 1


def load_inputs(w, ha, W, zero=False):
    """Inputs resident in HBM.  One-batch workloads are drawn on the host from the numpy stream the parity tests use
    (workloads.make_inputs, seed = w.seed), so bench and parity test see the same tensors; the B = 2 720p layers
    (1.9 GB each) are drawn on the device by the generator their parity test uses (workloads.make_inputs_on_device)."""
    if w.B == 1:
        q, k, v, fq, fk = ha.to_device(W.make_inputs(w), "cuda:0")
    else:
        q, k, v, fq, fk = ha.device_inputs(w, "cuda:0")
    if zero:
        q.zero_(), k.zero_(), v.zero_()
    if w.R == 1 and not w.local_window:
        fq = fk = None
    return q, k, v, fq, fk


def query_kernel_flops(w, W):
    """Algorithmic flops of the fused query kernel: 4 d per (query, softmax key) pair, the phi_q MLP and the contraction
    with the state (the latter two only when the kernel evaluates phi_q itself)."""
    n_l = w.N if w.local_window > 0 else w.n_linear
    layered = n_l > 0 and (w.d_mid or not ((w.d_hidden == w.d and w.d_feat == w.d) or (w.d_hidden == 256 and w.d_feat == 256)))
    fl = 4.0 * w.d * W.softmax_pairs(w)
    if n_l > 0 and not layered:
        fl += 2.0 * w.N * (w.d * w.d_hidden + w.d_hidden * w.d_feat) + 2.0 * w.N * w.d_feat * w.d + 2.0 * w.N * w.d_feat
    return w.B * w.H * fl


def mfma_probe_rates(ha, torch, dev):
    """Sustained matrix-core rate of this device next to the published peak: a kernel of nothing but MFMA instructions,
    run for a few hundred ms so that power management settles; operand values matter (zero operands keep the clock at
    its ceiling, random ones do not).  Recorded beside every figure so that runs on different boxes can be compared."""
    sink = torch.empty(torch.cuda.get_device_properties(0).multi_processor_count * 512, device=dev)
    out = {}
    for name, rnd in (("zero_operands", False), ("random_operands", True)):
        ha.hybrid_attn_mfma_probe(rnd, 20000, 20, sink)          # settle
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = ha.hybrid_attn_mfma_probe(rnd, 20000, 60, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name + "_tflops"] = fl * 60 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # the zero-operand probe runs at the clock ceiling: its rate over the per-clock width gives that clock
    out["clock_ghz_zero_operands"] = out["zero_operands_tflops"] * 1e12 / (256 * 4096) / 1e9
    out["clock_ghz_random_operands"] = out["random_operands_tflops"] * 1e12 / (256 * 4096) / 1e9
    return out


def settle_clocks(torch, step, batch=10, max_steps=200, tol=0.005):
    """Untimed steps until the GPU has left its idle clock state.  A process that has just generated its inputs finds
    the GPU idle, and the shader clock needs some tens of milliseconds of load to come up: the first five forwards at
    480p/81f take 1.66 ms, the next twenty 1.40 ms, every later one 1.35 ms (one box, 600 forwards in a row).  A loop
    of forwards (a 30-layer stack, a sampler's steps) runs at the last figure, so that is the state the timed region
    starts in: batches of `batch` steps until two batches in a row take the same time within `tol`, at most
    `max_steps` steps.  Returns the number of steps run (reported in the JSON line)."""
    prev, n = None, 0
    while n < max_steps:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(batch):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n += batch
        if prev is not None and abs(dt - prev) <= tol * prev:
            break
        prev = dt
    return n


def time_forward(ha, torch, step, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations.  During the timed steps the
    library records one pair of HIP events around the dominant kernel on the stream it is launched on (the light tap);
    returns (wall ms per step, mean kernel ms, sorted per-step kernel ms)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ha.hybrid_attn_profile_enable(-steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms = [ha.hybrid_attn_profile_read(i)[3] for i in range(steps)]
    ha.hybrid_attn_profile_enable(0)
    return elapsed * 1e3 / steps, sum(kernel_ms) / len(kernel_ms), sorted(kernel_ms)


def graph_replay_ms(torch, step_on_current_stream, steps):
    """The same step captured once into a HIP graph and replayed `steps` times (the forward is a fixed sequence of
    launches with no allocation, no host synchronisation and no memset): ms per replay.  A separate pass behind the
    timed region; the headline stays the eager figure."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step_on_current_stream()                      # warm-up on a side stream, as capture requires
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step_on_current_stream()
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def stage_breakdown(ha, torch, step, steps):
    """A second, untimed-for-the-headline pass with the full tap (five event records per forward): mean stage ms."""
    ha.hybrid_attn_profile_enable(steps)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    rows = [ha.hybrid_attn_profile_read(i) for i in range(steps)]
    ha.hybrid_attn_profile_enable(0)
    mean = [sum(r[i] for r in rows) / len(rows) for i in range(5)]
    fwd = sorted(r[4] for r in rows)
    return mean, fwd


def stack_mode(args, ha, W, torch):
    """The 720p / 81-frame stack: 30 layers with B = 2 (classifier-free guidance), rates cycling 16, 8, 4, every layer
    with its own seeded q, k, v and feature maps (seed 1000 + l), all resident in HBM (56 GB); one step = one pass over
    the 30 layers; tokens/s = B N 30 / t."""
    base = W.WAN_720P_81F_CFG
    dev = "cuda:0"
    layers = []
    for l in range(W.STACK_LAYERS):
        w = W.replace(base, R=W.STACK_RATES[l % len(W.STACK_RATES)], seed=1000 + l)
        q, k, v, fq, fk = ha.device_inputs(w, dev)
        layers.append((w, q, k, v, fq, fk, torch.empty_like(q)))
    ws_bytes = max(ha.hybrid_attn_workspace_bytes(ha.make_problem(L[1], L[0].R, L[0].block_size, L[0].scale), L[4], L[5]) for L in layers)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def run_stack():
        for (w, q, k, v, fq, fk, out) in layers:
            ha.hybrid_attn_forward(q, k, v, fq, fk, w.R, w.block_size, w.scale, out=out, workspace=ws, stream=stream)

    for _ in range(args.warmup):
        run_stack()
    torch.cuda.synchronize()
    n_l = len(layers)
    ha.hybrid_attn_profile_enable(-n_l * args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_stack()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    k_ms = [ha.hybrid_attn_profile_read(i)[3] for i in range(n_l * args.steps)]
    ha.hybrid_attn_profile_enable(0)
    for L in layers:
        assert torch.isfinite(L[6][:, :, ::997].float()).all().item(), "non-finite output"
    ms_per_step = elapsed * 1e3 / args.steps
    flops = sum(W.algorithmic_flops(L[0]) for L in layers)
    kflops = sum(query_kernel_flops(L[0], W) for L in layers)
    kernel_ms_per_stack = sum(k_ms) / args.steps
    per_rate = {}
    for i, ms in enumerate(k_ms):
        per_rate.setdefault(str(layers[i % n_l][0].R), []).append(ms)
    achieved = kflops / (kernel_ms_per_stack * 1e-3) / 1e12
    probe = None if args.no_mfma_probe else mfma_probe_rates(ha, torch, dev)
    rec = {
        "metric": "hybrid-attention fwd tokens/s", "value": base.B * base.N * n_l / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "wan1.3b_720p_81f_cfg2 x 30 layers", "B": base.B, "H": base.H, "N": base.N, "d_head": base.d,
                   "io_dtype": base.dtype, "layers": n_l, "hybrid_rates_R": list(W.STACK_RATES), "block_size": base.block_size,
                   "feature_map": f"{base.d}->{base.d_hidden}->{base.d_feat}, P={base.poly_degree}", "layer_seeds": "1000 + l",
                   "step": "one pass over the 30 layers"},
        "tflops": flops / (ms_per_step * 1e-3) / 1e12,
        "pct_bf16_mfma_peak": 100.0 * flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "query_kernel_ms_by_rate": {r: sum(v) / len(v) for r, v in per_rate.items()},
        "roofline": {"bound": "mfma", "kernel": "query_kernel (all 30 layers)", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "kernel_ms": kernel_ms_per_stack, "traffic": None,
                     "traffic_source": "not profiled for this workload",
                     "kernel_ms_source": "HIP events the library records around the kernel's launch on its stream, the timed steps of this run, summed over the 30 layers"},
    }
    if probe:
        rec["mfma_probe"] = probe
        rec["roofline"]["frac_of_sustained_mfma_rate"] = achieved / probe["random_operands_tflops"]
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline_extrapolated(layers[:3], W, torch)
    print(json.dumps(rec), flush=True)


def cpu_baseline_extrapolated(layers, W, torch):
    """The stack is 317 TFLOP of fp64 for the oracle: far beyond a bounded sample.  For one layer of each rate
    (16, 8, 4) and one (batch, head) pair the oracle's state pass is run in full and its per-query part on a sample of
    rows; t_layer = B H (t_state + t_row N), the stack is ten times the three layers.  EXTRAPOLATED, and labelled so."""
    from oracle import hybrid_attn_oracle as O
    t_stack, notes = 0.0, []
    for (w, q, k, v, fq, fk, _) in layers:
        qh, kh, vh = (t[0, 0].float().cpu().numpy() for t in (q, k, v))
        oq, ok = (O.FeatureMap(m.w1.float().cpu().numpy(), m.b1.cpu().numpy(), m.w2.float().cpu().numpy(), m.b2.cpu().numpy(),
                               m.poly_degree) for m in (fq, fk))
        t0 = time.perf_counter()
        O.linear_state(kh, vh, ok, 0, w.R)
        t_state = time.perf_counter() - t0
        rows = W.sample_rows(w, 256)
        t0 = time.perf_counter()
        O.hybrid_attn_head(qh, kh, vh, oq, ok, 0, w.R, w.scale, rows=rows)
        t_rows = time.perf_counter() - t0 - t_state          # hybrid_attn_head recomputes the state
        t_layer = w.B * w.H * (t_state + max(t_rows, 0.0) / len(rows) * w.N)
        notes.append(f"R={w.R}: state {t_state:.2f} s, {len(rows)} rows {t_rows:.2f} s -> {t_layer:.0f} s per layer")
        t_stack += t_layer * (W.STACK_LAYERS // len(W.STACK_RATES))
    w = layers[0][0]
    return {"value": w.B * w.N * W.STACK_LAYERS / t_stack, "unit": "tokens/s", "cores": host_threads(), "cpu_model": cpu_model(),
            "kind": "oracle", "extrapolated": True,
            "sample": "EXTRAPOLATED: per rate one (batch, head) pair, full fp64 state pass + per-query part on sampled rows, scaled "
                      "to B H pairs, N rows and 10 layers per rate; " + "; ".join(notes) + f"; stack {t_stack:.0f} s"}


def rate_sweep_mode(args, ha, W, torch):
    """Cost against the softmax fraction r = 1/R (Sec. 3.3: the per-block rates the knapsack chooses from; Fig. "teaser":
    cost against length): the 480p / 81-frame shape at R in {0, 16, 8, 4, 2, 1} and the 1024-token fp32 case at
    R in {0, 8, 4, 2, 1}; least-squares fit t(r) = t0 + t1 r over the r > 0 points.  Writes one JSON document."""
    dev = "cuda:0"
    probe = mfma_probe_rates(ha, torch, dev)
    doc = {"command": "python bench.py --rate-sweep --steps %d --warmup %d" % (args.steps, args.warmup),
           "mfma_probe": probe, "sweeps": {}}
    for name, base, rates in (("wan1.3b_480p_81f", W.WAN_480P_81F, (0, 16, 8, 4, 2, 1)), ("tiny", W.TINY, W.RATE_SWEEP)):
        inp = ha.to_device(W.make_inputs(base), dev)
        rows = []
        for R in rates:
            w = W.with_rate(base, R)
            q, k, v = inp[:3]
            fq, fk = (None, None) if R == 1 else inp[3:]
            ws = torch.empty(ha.hybrid_attn_workspace_bytes(ha.make_problem(q, R, w.block_size, w.scale), fq, fk), dtype=torch.uint8, device=dev)
            out = torch.empty_like(q)
            stream = torch.cuda.current_stream()

            def step():
                ha.hybrid_attn_forward(q, k, v, fq, fk, R, w.block_size, w.scale, out=out, workspace=ws, stream=stream)
            settle_clocks(torch, step)
            ms, kernel_ms, _ = time_forward(ha, torch, step, args.steps, args.warmup)
            fl = W.algorithmic_flops(w)
            row = {"R": R, "r": (1.0 / R if R else 0.0), "forward_ms": ms, "query_kernel_ms": kernel_ms, "algorithmic_gflop": fl / 1e9,
                   "tflops": fl / (ms * 1e-3) / 1e12, "pct_bf16_mfma_peak": 100.0 * fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                   "tokens_per_s": w.B * w.N / (ms * 1e-3)}
            if R == 0:
                row["hbm_gbs_on_algorithmic_bytes"] = W.algorithmic_bytes(w) / (ms * 1e-3) / 1e9
            rows.append(row)
            print(f"  {name} R={R}: {ms:.4f} ms", file=sys.stderr, flush=True)
        pos = [r for r in rows if r["R"] > 0]
        n = len(pos)
        sx, sy = sum(r["r"] for r in pos), sum(r["forward_ms"] for r in pos)
        sxx, sxy = sum(r["r"] ** 2 for r in pos), sum(r["r"] * r["forward_ms"] for r in pos)
        t1 = (n * sxy - sx * sy) / (n * sxx - sx * sx)
        t0 = (sy - t1 * sx) / n
        full = next(r["forward_ms"] for r in rows if r["R"] == 1)
        for r in rows:
            r["speedup_over_r1"] = full / r["forward_ms"]
        doc["sweeps"][name] = {"shape": {"B": base.B, "H": base.H, "N": base.N, "d_head": base.d, "io_dtype": base.dtype,
                                         "block_size": base.block_size}, "points": rows,
                               "fit_ms": {"t0": t0, "t1": t1, "model": "t(r) = t0 + t1 r, least squares over r > 0",
                                          "max_rel_residual": max(abs(t0 + t1 * r["r"] - r["forward_ms"]) / r["forward_ms"] for r in pos)},
                               "linear_floor_ms_r0": next(r["forward_ms"] for r in rows if r["R"] == 0)}
    doc["mfma_probe_after"] = mfma_probe_rates(ha, torch, dev)
    text = json.dumps(doc, indent=1)
    if args.out:
        os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
        open(args.out, "w").write(text + "\n")
    print(json.dumps(doc), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="wan_480p_81f", choices=["tiny", "wan_480p_81f", "wan_480p_161f", "wan_720p_81f_cfg"])
    ap.add_argument("--rate", type=int, default=None, help="override the hybrid rate R (0 = pure linear, 1 = full softmax)")
    ap.add_argument("--block-size", type=int, default=None)
    ap.add_argument("--phi-width", type=int, default=None,
                    help="hidden and output width of both feature maps (default: the workload's d -> d -> d; 256, 384, 512 "
                         "are the two-layer rows P = 2, 3, 4 of Tab. phi at d = 128, 768 the width of its P = 6 row)")
    ap.add_argument("--phi-layers", type=int, default=2, choices=[2, 3],
                    help="MLP depth of both feature maps; 3 adds a hidden layer of the same width (Tab. phi, P = 6 row)")
    ap.add_argument("--split-granularity", type=int, default=0, metavar="G",
                    help="variant of the token split: groups of G consecutive tokens, every R-th group softmax tokens")
    ap.add_argument("--causal-chunk", type=int, default=0, metavar="C",
                    help="chunk-causal variant: a query sees its own and all earlier chunks of C tokens (multiple of 2 * block size)")
    ap.add_argument("--local-window", type=int, default=0, metavar="W",
                    help="local-window variant: softmax over the query's tile and W tokens on either side (multiple of 2 * block "
                         "size), linear attention over every other token; sets the rate to 0")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack", action="store_true",
                    help="the 720p / 81-frame stack: 30 layers, B = 2, rates cycling 16, 8, 4, per-layer seeds 1000 + l; one step = "
                         "one pass over the stack; prints one JSON line about it instead of the headline line")
    ap.add_argument("--rate-sweep", action="store_true",
                    help="forward time against the softmax fraction r = 1/R at the 480p / 81-frame shape and at the 1024-token "
                         "case, with the fit t0 + t1 r; prints (and with --out writes) one JSON document")
    ap.add_argument("--out", default=None, help="with --rate-sweep: file to write the JSON document to")
    ap.add_argument("--select-rates", type=float, default=None, metavar="BETA",
                    help="block-rate selection mode (Sec. 3.3): measure the cost of one layer at R in {1, 2, 4, 8}, draw "
                         "synthetic per-layer errors, solve the knapsack for a budget of BETA x the all-softmax stack, "
                         "run the selected 30-layer stack and print one JSON line about it instead of the headline line")
    ap.add_argument("--measured-errors", action="store_true",
                    help="with --select-rates: take e_{l,R} from the value-distillation loss (Eq. vd_loss) of layer l's own "
                         "seeded random feature maps on the shared synthetic q, k, v instead of drawing it")
    ap.add_argument("--distill-step", action="store_true",
                    help="time one student update of the distillation loop (Sec. 3.3, Alg. 1: student forward, loss, gradient "
                         "of the feature maps on the cached teacher output) and print one JSON line about it instead of the "
                         "headline line")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="all-zero q, k, v: NOT a benchmark, a power / clock experiment (same instruction stream, idle data wires)")
    ap.add_argument("--no-cold-cache", action="store_true", help="skip the extra forwards with flushed caches")
    ap.add_argument("--graph", action="store_true",
                    help="one more pass that replays the forward from a HIP graph (forward_ms_hip_graph_replay; on this "
                         "runtime a replay is no faster than the three eager launches: 1.38 vs 1.36 ms, 37 vs 39 us at 1024 tokens)")
    ap.add_argument("--no-clock-settle", action="store_true",
                    help="skip the untimed steps that bring the GPU out of its idle clock state before the warm-up")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the matrix-core probe (sustained MFMA-only rate of this device, zero and random operands)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference kernel for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_24899_amd import hybrid_attn as ha
    from paper_2509_24899_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if args.stack:
        stack_mode(args, ha, W, torch)
        return
    if args.rate_sweep:
        rate_sweep_mode(args, ha, W, torch)
        return

    w = {"tiny": W.TINY, "wan_480p_81f": W.WAN_480P_81F, "wan_480p_161f": W.WAN_480P_161F,
         "wan_720p_81f_cfg": W.WAN_720P_81F_CFG}[args.workload]
    if args.rate is not None:
        w = W.with_rate(w, args.rate)
    if args.block_size is not None:
        w = W.replace(w, block_size=args.block_size)
    if args.phi_width is not None:
        # Tab. "phi": D' = d channels per slice, so a map of width P d has polynomial degree P
        w = W.replace(w, d_hidden=args.phi_width, d_feat=args.phi_width,
                      poly_degree=args.phi_width // w.d if args.phi_width % w.d == 0 else w.poly_degree)
    if args.phi_layers == 3:
        w = W.replace(w, d_mid=w.d_hidden)
    if args.split_granularity > 1:
        w = W.replace(w, split_granularity=args.split_granularity)
    if args.causal_chunk > 0:
        w = W.replace(w, causal_chunk=args.causal_chunk)
    if args.local_window > 0:
        w = W.replace(w, R=0, local_window=args.local_window)

    # synthetic inputs, seeded, resident in HBM before the timed region
    if args.distill_step or args.select_rates is not None:
        q, k, v, fq, fk = load_inputs(W.with_rate(w, w.R if w.R != 1 else 4), ha, W)     # these modes need feature maps at every rate
        if args.distill_step:
            distill_step_mode(args, w, ha, torch, q, k, v, fq, fk)
        else:
            rate_selection_mode(args, w, ha, W, torch, q, k, v, fq, fk, torch.empty_like(q))
        return
    q, k, v, fq, fk = load_inputs(w, ha, W, zero=args.zero_inputs)
    prob = ha.make_problem(q, w.rate, w.block_size, w.scale)
    ws = torch.empty(ha.hybrid_attn_workspace_bytes(prob, fq, fk), dtype=torch.uint8, device=dev)
    out = torch.empty_like(q)
    stream = torch.cuda.current_stream()

    def step():
        ha.hybrid_attn_forward(q, k, v, fq, fk, w.rate, w.block_size, w.scale, out=out, workspace=ws, stream=stream)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    settle_steps = 0 if args.no_clock_settle else settle_clocks(torch, step)
    ms_per_step, kernel_ms, kernel_sorted = time_forward(ha, torch, step, args.steps, args.warmup)
    assert torch.isfinite(out.float()).all().item(), "non-finite output"
    mean, fwd_sorted = stage_breakdown(ha, torch, step, args.steps)

    # cold-cache forwards: a 512 MiB fill between forwards evicts L2 and the 256 MiB Infinity Cache, so inputs,
    # weights and workspace come from HBM (matters for the HBM-bound r = 0 point; the timing is the forward's
    # own event pair, the fill lies outside it)
    cold_sorted = None
    if not args.no_cold_cache:
        n_cold = min(10, args.steps)
        flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        ha.hybrid_attn_profile_enable(n_cold)
        for i in range(n_cold):
            flush.fill_(i & 0xFF)
            step()
        torch.cuda.synchronize()
        cold_sorted = sorted(ha.hybrid_attn_profile_read(i)[4] for i in range(n_cold))
        ha.hybrid_attn_profile_enable(0)
        del flush

    graph_ms = None
    if args.graph:
        def step_on_current_stream():
            ha.hybrid_attn_forward(q, k, v, fq, fk, w.rate, w.block_size, w.scale, out=out, workspace=ws,
                                   stream=torch.cuda.current_stream())
        graph_ms = graph_replay_ms(torch, step_on_current_stream, args.steps)

    mfma_probe = None if args.no_mfma_probe else mfma_probe_rates(ha, torch, dev)

    flops = W.algorithmic_flops(w)
    n_s = w.N if w.local_window > 0 else w.n_softmax
    events_note = "HIP events the library records around the kernel's launch on its stream, mean over the timed steps of this run"
    if n_s > 0:
        # dominant kernel: the fused query kernel
        achieved = query_kernel_flops(w, W) / (kernel_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "query_kernel", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "kernel_ms": kernel_ms, "kernel_ms_source": events_note, "traffic": None,
                    "traffic_source": "this workload has not been profiled"}
    else:
        # r = 0: no softmax keys, the whole forward is bound by HBM; the clock is the wall clock over the timed steps
        by = W.algorithmic_bytes(w)
        achieved = by / (ms_per_step * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "whole forward (r = 0): state pass + state reduction + query-side kernel", "achieved": achieved,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "kernel_ms": ms_per_step,
                    "kernel_ms_source": "wall clock over the timed steps of this run (the forward is three launches)",
                    "query_side_kernel_ms": kernel_ms, "traffic": None, "traffic_source": "this workload has not been profiled"}
    # HBM bytes per launch of the dominant kernel: NOT measured in this run; read from the committed summary of the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this same command (null when this workload has not been profiled)
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file) and w.d_hidden == w.d and w.d_feat == w.d and w.split_granularity <= 1 and not w.causal_chunk and not w.local_window:   # profiled with the d -> d -> d maps
        t = json.load(open(traffic_file)).get(f"{w.name}_R{w.R}_bs{w.block_size}")
        if t:
            roofline["traffic"] = t["read_bytes"] + t["written_bytes"]
            roofline["traffic_detail"] = t
            roofline["traffic_source"] = ("profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this command, scaled by a "
                                          "1 GiB copy in the same process; committed with the profile summaries, not measured in this run")

    if mfma_probe and roofline["bound"] == "mfma":
        roofline["frac_of_sustained_mfma_rate"] = roofline["achieved"] / mfma_probe["random_operands_tflops"]
    rec = {
        "metric": "hybrid-attention fwd tokens/s", "value": w.B * w.N / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "clock_settle_steps": settle_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if not args.zero_inputs else "all-zero q, k, v (clock experiment, not a benchmark)",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d_head": w.d, "io_dtype": w.dtype,
                   "hybrid_rate_R": w.R, "r": (1.0 / w.R if w.R else 0.0), "block_size": w.block_size,
                   **({"split_granularity": w.split_granularity} if w.split_granularity > 1 else {}),
                   **({"causal_chunk": w.causal_chunk} if w.causal_chunk else {}),
                   **({"local_window": w.local_window} if w.local_window else {}),
                   "feature_map": (f"{w.d}->{w.d_hidden}->{w.d_mid}->{w.d_feat}" if w.d_mid else f"{w.d}->{w.d_hidden}->{w.d_feat}")
                   + f", P={w.poly_degree}",
                   "inputs": "workloads.make_inputs (numpy stream, seed %d): the tensors of the parity test at this shape" % w.seed if w.B == 1
                             else "workloads.make_inputs_on_device (torch generator, seed %d)" % w.seed},
        "tflops": flops / (ms_per_step * 1e-3) / 1e12,
        "pct_bf16_mfma_peak": 100.0 * flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "query_kernel_ms_median": kernel_sorted[len(kernel_sorted) // 2], "query_kernel_ms_min": kernel_sorted[0],
        "forward_ms_cold_cache_median": cold_sorted[len(cold_sorted) // 2] if cold_sorted else None,
        "forward_ms_hip_graph_replay": graph_ms,
        "stage_ms": {"compact": mean[0], "state": mean[1], "wprep_q": mean[2], "query": mean[3], "forward": mean[4],
                     "forward_median": fwd_sorted[len(fwd_sorted) // 2], "forward_min": fwd_sorted[0],
                     "source": "a second pass of the same steps, outside the timed region, with an event record between all stages "
                               "(the records themselves cost the stream about 15 us per forward)"},
        "roofline": roofline,
    }
    if mfma_probe:
        rec["mfma_probe"] = mfma_probe
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
