#!/usr/bin/env python3
"""Benchmark of the Symi MoE hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input already
resident in HBM: route -> dispatch -> expert forward -> combine -> combine backward ->
expert backward -> dispatch backward -> route backward -> place (next placement) ->
Adam on this GPU's 1/N shard + write into the next placement's replica slots.  The
default workload is config c5 of the benchmark spec, the largest one (bf16, E=128, top-8,
d=4096, f=2048, T=65536, 256 slots, N=32, near-uniform Zipf-0.5 popularity); --config
picks another (c2 and c4 cycle through their 10 / 20 iterations).  All N optimizer
partitions step during the warm-up, so that the timed steps start from the method's
state; a timed step runs this GPU's partition only (the other N-1 live on other GPUs).

Prints ONE JSON line: whole-job tokens/s, the roofline of the dominant kernel (from HIP
events recorded around every launch of the timed steps run a second time), the step
times and Adam rates of the other four configs (`other_configs`), and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0     # dense bf16 MFMA
FP32_VEC_PEAK_TF = 157.3       # fp32 vector FMA


def kernel_work(c, w, nonempty_slots, grad_classes):
    """Algorithmic (flops, bytes) of one launch of each kernel for workload c."""
    T, E, k, d, f, S, N = c.T, c.E, c.k, c.d, c.f, c.S_tot, c.N
    A = T * k
    Sn = nonempty_slots
    Eg = grad_classes      # classes whose weight gradient is written by the backward and read by Adam
    nblk = (A + 1023) // 1024
    per = 3 * d * f // N
    return {
        "route": (0, T * (4 * E + 8 * k) + 4 * E),
        "route_bwd": (0, T * (8 * E + 12 * k)),
        "chunk_count": (0, 4 * A + 4 * nblk * E),
        "chunk_scan": (0, 8 * nblk * E),
        "chunk_rank": (0, 12 * A + 4 * nblk * E),
        "gather_rows": (0, T * d * w + A * d * w + 4 * A),
        "gemm_fwd1": (2 * A * d * 2 * f, Sn * 2 * f * d * w + A * d * w + A * 3 * f * w),
        "gemm_fwd2": (2 * A * f * d, Sn * d * f * w + A * f * w + A * d * w),
        "gemm_bwd_dh": (2 * A * d * f, Sn * d * f * w + A * d * w + 4 * A * f * w),
        "gemm_bwd_dx": (2 * A * 2 * f * d, Sn * 2 * f * d * w + A * 2 * f * w + A * d * w),
        "gemm_wgrad2": (2 * A * d * f, A * d * w + A * f * w + Eg * d * f * 4),
        "gemm_wgrad1": (2 * A * 2 * f * d, A * 2 * f * w + A * d * w + Eg * 2 * f * d * 4),
        "combine": (0, A * d * w + T * d * w + 8 * A),
        "combine_bwd": (0, T * d * w + 2 * A * d * w + 12 * A),
        "dispatch_bwd": (0, A * d * w + T * d * w + 4 * A),
        "adam_to_replicas": (0, E * per * 24 + Eg * per * 4 + S * per * w),
    }


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` as measured with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size); the figures and the
    commands that produced them are kept in profiles/hbm_traffic.json.  None if absent."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            return json.load(fh)[workload][kernel]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def survival(args):
    """Token survival (Sec. 3.4, Sec. 5.2) per iteration of a config under capacity_factor,
    for the placement that mimics the previous iteration and for the static uniform one.
    Integer stages only (route, place, capacity-limited dispatch); one JSON line per iteration."""
    import torch
    import paper_2504_19925_amd as symi
    import workloads as wl
    import harness as Hn

    c = wl.get_config(args.config)
    cfg = Hn.make_ctx(c)
    dev = "cuda"
    i32 = dict(dtype=torch.int32, device=dev)
    ws = torch.empty(symi.symi_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    X = torch.zeros(c.T, c.d, dtype=cfg.torch_dtype, device=dev)
    Xp = torch.empty(c.A, c.d, dtype=cfg.torch_dtype, device=dev)
    idx = torch.empty(c.T, c.k, **i32)
    gate = torch.empty(c.T, c.k, dtype=torch.float32, device=dev)
    hist = torch.empty(c.E, **i32)
    counts, placement, first = torch.empty(c.E, **i32), torch.empty(c.S_tot, **i32), torch.empty(c.E + 1, **i32)
    roa, aor, off = torch.empty(c.A, **i32), torch.empty(c.A, **i32), torch.empty(c.S_tot + 1, **i32)
    cap = symi.symi_slot_capacity(cfg, args.survival)
    prev = torch.zeros(c.E, **i32)
    for it in range(max(c.iters, 1)):
        logits = wl.make_logits(c, it).to(dev)
        symi.symi_route(cfg, logits, idx, gate, hist)
        out = {"workload": c.name, "iteration": it, "capacity_factor": args.survival, "slot_capacity": cap}
        for mode, pop in (("adaptive", prev), ("uniform", torch.zeros(c.E, **i32))):
            symi.symi_place(cfg, pop, counts, placement, first)
            symi.symi_dispatch_capacity(cfg, cap, X, idx, hist, counts, first, roa, aor, off, Xp, ws)
            out["survival_" + mode] = round(int(off[-1]) / c.A, 5)
        print(json.dumps(out))
        prev = hist.clone()


def extras(args):
    """Kernel times of the entry points around the core path on --config: the router GEMM and
    its backward, and the replica gradient path as the paper draws it (per-slot weight
    gradients + intra-rank all-reduce) next to the fused per-class one.  One JSON line."""
    import torch
    import paper_2504_19925_amd as symi
    import workloads as wl
    import harness as Hn

    c = wl.get_config(args.config)
    st = Hn.State(c, flags=symi.CTX_TIMING | symi.CTX_NO_OVERLAP)
    s, cfg = st, st.ctx
    X, logits, dY = Hn.draw_inputs(c, 0)
    st.place_current()
    st.forward(X, logits)
    st.backward(dY, logits)
    st.hist_prev.copy_(st.hist)          # placement that mimics this popularity: replicated classes
    st.place_current()
    st.forward(X, logits)
    Wr, b = wl.make_router(c, 0, "cuda")
    lg = torch.empty(c.T, c.E, dtype=torch.float32, device="cuda")
    dWr = torch.empty(c.E, c.d, dtype=torch.float32, device="cuda")
    db = torch.empty(c.E, dtype=torch.float32, device="cuda")
    g1 = torch.empty(c.S_tot, 2 * c.f, c.d, dtype=torch.float32, device="cuda")
    g2 = torch.empty(c.S_tot, c.d, c.f, dtype=torch.float32, device="cuda")

    def router():
        symi.symi_router_fwd(cfg, X, Wr, b, lg)
        symi.symi_router_bwd(cfg, X, Wr, s.dlogits, dWr, db, s.dX, s.ws)

    def fused():
        symi.symi_expert_bwd(cfg, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s, s.W2s,
                             s.dXp, s.dW1, s.dW2, s.ws)

    def drawn():
        symi.symi_expert_bwd_slots(cfg, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s,
                                   s.W2s, s.dXp, g1, g2, s.ws)
        symi.symi_replica_allreduce(cfg, s.first_slot, 1.0, g1, g2)

    symi.symi_combine_bwd(cfg, dY, s.Yp, s.row_of_assign, s.gate, s.dYp, s.dgate)
    out = {"workload": c.name, "unit": "us per call, all launches of a kernel id summed", "steps": args.steps}
    for fn in (router, fused, drawn):
        for _ in range(2):
            fn()
        Hn.sync()
        symi.symi_timing_reset(cfg)
        for _ in range(args.steps):
            fn()
        Hn.sync()
        got = {}
        for kid in range(symi.symi_kernel_count()):
            ms, n = symi.symi_timing_read(cfg, kid)
            if n:
                got[symi.symi_kernel_name(kid)] = round(ms / args.steps * 1e3, 1)
        got["total"] = round(sum(got.values()), 1)
        out[fn.__name__] = got
    w = 2 if c.dtype == "bf16" else 4
    out["router_floor_us_at_8TBps"] = {"fwd": round(c.T * c.d * w / 8e6, 1),
                                       "dx": round((2 * c.T * c.d * w + 4 * c.T * c.E) / 8e6, 1),
                                       "dw": round((c.T * c.d * w + 4 * c.T * c.E) / 8e6, 1)}
    print(json.dumps(out))


def ceilings(args):
    """What this GPU sustains with the instruction and access mixes of the hot path's kernels
    (in-bounds microbenchmarks of libsymi_ceilings.so and of torch's fill / copy); one JSON line.
    Every figure is the average of `reps` back-to-back launches between two events on the
    launch stream."""
    import ctypes
    import torch

    path = os.path.join(ROOT, "paper_2504_19925_amd", "libsymi_ceilings.so")
    if not os.path.exists(path):
        raise SystemExit(f"{path} not found: build it with `python -m paper_2504_19925_amd.build`")
    L = ctypes.CDLL(path)
    vp, ci, cll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
    L.symi_ceiling_mfma.argtypes = [vp, vp, ci, ci, vp]
    L.symi_ceiling_gemm_loop.argtypes = [ci, vp, vp, vp, ci, ci, ci, cll, cll, vp]
    L.symi_ceiling_adam_streams.argtypes = [ci, vp, vp, vp, vp, vp, vp, cll, ci, vp]
    torch.cuda.set_device(0)
    stream = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def call(rc):
        if rc != 0:
            raise SystemExit(f"ceiling launch failed ({rc})")

    out = {"unit_note": "TFLOP/s for mfma and gemm_loop, GB/s for the streams", "reps": args.steps}
    g = torch.Generator(device="cuda").manual_seed(1)
    # ---- MFMA from registers: 1024 workgroups (4 per CU), 4000 x 16 MFMAs per wavefront
    blocks, iters = 1024, 4000
    res = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    for name, ops in (("random", torch.randn(blocks * 256 * 16, generator=g, device="cuda").to(torch.bfloat16)),
                      ("zeros", torch.zeros(blocks * 256 * 16, dtype=torch.bfloat16, device="cuda"))):
        s = timed(lambda: call(L.symi_ceiling_mfma(ptr(ops), ptr(res), blocks, iters, stream())), 5)
        out["mfma_regs_" + name] = round(blocks * 4 * iters * 16 * 32768.0 / s / 1e12, 1)
    # ---- the GEMM's reduction loop on C = A B^T, 8192 x 8192 x 4096
    M = N = 8192
    K = 4096
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    names = {0: "gemm_loop", 1: "gemm_loop_no_loads", 2: "gemm_loop_no_lds_reads", 3: "gemm_loop_no_mfma"}
    for dname in ("random", "zeros"):
        if dname == "random":
            A = torch.randn(M + 256, K, generator=g, device="cuda").to(torch.bfloat16)
            B = torch.randn(N + 256, K, generator=g, device="cuda").to(torch.bfloat16)
        else:
            A = torch.zeros(M + 256, K, dtype=torch.bfloat16, device="cuda")
            B = torch.zeros(N + 256, K, dtype=torch.bfloat16, device="cuda")
        for variant, name in names.items():
            s = timed(lambda: call(L.symi_ceiling_gemm_loop(variant, ptr(A), ptr(B), ptr(C), M, N, K,
                                                            A.numel(), B.numel(), stream())), args.steps)
            out[f"{name}_{dname}"] = round(2.0 * M * N * K / s / 1e12, 1)   # MFMA-equivalent rate
        # the vendor library's kernel for the same product (torch.matmul -> hipBLASLt), and for a
        # deeper one: what a plain bf16 GEMM reaches on this part with this data
        s = timed(lambda: torch.matmul(A[:M], B[:N].t(), out=C), args.steps)
        out[f"vendor_gemm_8192x8192x4096_{dname}"] = round(2.0 * M * N * K / s / 1e12, 1)
        del A, B
    del C
    # ---- the Adam step's streams on c2's shard (100.7 M parameters, 1.5 replicas per parameter)
    n = 100663296
    gr = torch.randn(n, generator=g, device="cuda")
    w = torch.randn(n, generator=g, device="cuda")
    m = torch.zeros(n, device="cuda")
    v = torch.full((n,), 1e-4, device="cuda")
    s0 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    s1 = torch.empty(n // 2, dtype=torch.bfloat16, device="cuda")
    by = n * (16.0 + 12.0 + 3.0)
    for layout, lname in ((0, "8_per_thread"), (1, "lane_contiguous_x1"), (2, "lane_contiguous_x2"), (4, "lane_contiguous_x4")):
        for gs, gname in ((0, "one_pass"), (1, "grid_stride")):
            s = timed(lambda: call(L.symi_ceiling_adam_streams(layout, ptr(gr), ptr(w), ptr(m), ptr(v), ptr(s0), ptr(s1),
                                                               n, gs, stream())), args.steps)
            out[f"adam_streams_{lname}_{gname}"] = round(by / s / 1e9, 1)
    # ---- torch's own streaming kernels on the same buffers
    out["torch_fill"] = round(4.0 * n / timed(lambda: w.fill_(1.0), args.steps) / 1e9, 1)
    out["torch_copy"] = round(8.0 * n / timed(lambda: m.copy_(w), args.steps) / 1e9, 1)
    out["torch_add"] = round(12.0 * n / timed(lambda: torch.add(w, gr, out=m), args.steps) / 1e9, 1)
    print(json.dumps(out))


def calibrate_copy():
    """A plain copy of known size, to scale the HBM counters: 8 copies of 1 GiB."""
    import torch
    n = 1 << 29
    src = torch.ones(n, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(8):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": 2 * n, "copy_bytes_written": 2 * n, "copies": 8}))


def measure(c, args, steps, warmup):
    """Times `steps` steps of workload c after `warmup` untimed ones; returns the figures of
    the JSON line for that workload."""
    import torch
    import paper_2504_19925_amd as symi
    import harness as Hn

    flags = symi.CTX_NO_OVERLAP if args.no_overlap else 0
    # all N optimizer partitions are held and step during the warm-up (every slot is then
    # whole, as after the N ranks of the method); partition 0 is this GPU's
    st = Hn.State(c, shard=0, all_shards=True, flags=flags)
    st.active_grads = not args.dense_grads
    # second context for the per-kernel table: HIP events around every launch, one stream
    ctx_plain = st.ctx
    ctx_timed = Hn.make_ctx(c, 0, 1, symi.CTX_TIMING | symi.CTX_NO_OVERLAP)
    iters = max(c.iters, 1)
    inputs = [Hn.draw_inputs(c, it) for it in range(iters)]
    adam, _ = Hn.make_adam()
    st.place_current()            # placement of iteration 0 (uniform) + slot weights
    Hn.sync()

    def use(ctx):
        st.ctx = ctx
        st.opt[0] = (ctx,) + tuple(st.opt[0][1:])

    def step(i, shards=(0,)):
        X, logits, dY = inputs[i % iters]
        st.forward(X, logits)
        st.backward(dY, logits)
        st.optimizer(adam, shards=shards)
        st.advance()   # the placement computed in this step is the one the next step dispatches with

    def timed(n_steps, first):
        Hn.sync()
        t0 = time.perf_counter()
        for i in range(n_steps):
            step(first + i)
        Hn.sync()
        return (time.perf_counter() - t0) * 1e3 / n_steps

    def timed_graphs(n_steps, first):
        """The same n_steps steps replayed from HIP graphs: one graph per distinct step (the
        inputs cycle with period `iters`, the current/next placement buffers with period 2)."""
        import math
        period = math.lcm(2, iters)
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for j in range(min(period, n_steps)):
                g = torch.cuda.CUDAGraph()
                g.capture_begin()
                step(first + j)
                g.capture_end()
                graphs.append(g)
            if len(graphs) % 2:       # the captures swapped the buffer roles an odd number of times
                st.advance()
            Hn.sync()
            t0 = time.perf_counter()
            for j in range(n_steps):
                graphs[j % period].replay()
            Hn.sync()
            t1 = time.perf_counter()
        torch.cuda.current_stream().wait_stream(side)
        if n_steps % 2:               # the eager steps that follow start where the replays ended
            st.advance()
        del graphs
        return (t1 - t0) * 1e3 / n_steps

    for i in range(warmup):
        step(i, shards=None)
    # the timed region: the library as it ships, nothing but the K steps between two
    # synchronisations (no events: a pair around each of the ~20 launches of a step costs 6 % on
    # c2; the backward's two chains of products may share the chip on two streams)
    if args.graph:
        ms_per_step = timed_graphs(steps, warmup)
    else:
        ms_per_step = timed(steps, warmup)
    # per-kernel durations and the roofline come from the same steps run again through a context
    # that records HIP events around every launch and keeps one kernel at a time on the stream,
    # which is also what the committed rocprofv3 summary shows
    use(ctx_timed)
    step(warmup + steps)
    step(warmup + steps + 1)
    Hn.sync()
    symi.symi_timing_reset(ctx_timed)
    ms_serial = timed(steps, warmup)
    times = {}
    for kid in range(symi.symi_kernel_count()):
        ms, n = symi.symi_timing_read(ctx_timed, kid)
        if n:
            times[symi.symi_kernel_name(kid)] = (ms / n, n)
    symi.symi_timing_reset(ctx_timed)
    use(ctx_plain)
    w = 2 if c.dtype == "bf16" else 4

    # slots that actually hold rows (their weights are the ones a step must read)
    nonempty, active = [], []
    for i in range(iters):
        step(warmup + i)
        Hn.sync()
        so = st.slot_offsets.cpu()
        nonempty.append(int((so[1:] > so[:-1]).sum()))
        active.append(int((st.hist > 0).sum()))
    mean_nonempty = sum(nonempty) / len(nonempty)
    mean_active = sum(active) / len(active)

    work = kernel_work(c, w, mean_nonempty, c.E if args.dense_grads else mean_active)
    peak_tf = MFMA_BF16_PEAK_TF if c.dtype == "bf16" else FP32_VEC_PEAK_TF
    kernels = {}
    for name, (avg_ms, n) in times.items():
        entry = {"avg_us": round(avg_ms * 1e3, 2), "launches_per_step": round(n / steps, 2)}
        if name in work:
            fl, by = work[name]
            entry["GB/s"] = round(by / (avg_ms * 1e-3) / 1e9, 1)
            if fl:
                entry["TFLOP/s"] = round(fl / (avg_ms * 1e-3) / 1e12, 1)
        kernels[name] = entry
    gpu_ms = sum(avg * n for avg, n in times.values()) / steps
    fb = [k_ for k_ in times if k_ not in ("place", "adam_to_replicas")]
    fwd_bwd_ms = sum(times[k_][0] * times[k_][1] for k_ in fb) / steps

    dom = max((k_ for k_ in times if k_ in work), key=lambda k_: times[k_][0] * times[k_][1])
    fl, by = work[dom]
    avg_s = times[dom][0] * 1e-3
    t_hbm, t_mfma = by / (HBM_PEAK_GBS * 1e9), fl / (peak_tf * 1e12)
    if t_mfma > t_hbm:
        bound = "mfma" if c.dtype == "bf16" else "alu"
        roof = {"bound": bound, "achieved": round(fl / avg_s / 1e12, 2), "peak": peak_tf,
                "unit": "TFLOP/s", "frac": round(fl / avg_s / 1e12 / peak_tf, 4)}
    else:
        roof = {"bound": "hbm", "achieved": round(by / avg_s / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(by / avg_s / 1e9 / HBM_PEAK_GBS, 4)}
    roof.update({"kernel": dom, "avg_us": round(avg_s * 1e6, 2),
                 "measured": "HIP events around every launch, second pass of the same steps, one kernel at a time",
                 "traffic": measured_traffic(c.name, dom),
                 "algorithmic_bytes": by, "algorithmic_flops": fl})

    out = {
        "metric": "MoE layer fwd+bwd tokens/s; grouped-GEMM MFMA %; Adam+scatter HBM GB/s",
        "value": round(c.T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": f"{c.name}: {c.dtype} E={c.E} top-{c.k} d={c.d} f={c.f} T={c.T} "
                               f"S_tot={c.S_tot} N={c.N} (1 shard of {c.N}), {iters} iteration(s) cycled",
                   "step": "route+dispatch+expert_fwd+combine+backward+place+adam_to_replicas",
                   "weight_gradients": "all classes, zeros written and read for those without tokens"
                   if args.dense_grads else
                   "classes with tokens only (symi_expert_bwd_active + symi_adam_to_replicas_active: "
                   "same master weights, moments and slots, bit for bit)"},
        "roofline": roof,
        "fwd_bwd_tokens_per_s": round(c.T / (fwd_bwd_ms * 1e-3), 1),
        "gpu_kernel_ms_per_step": round(gpu_ms, 4),
        "ms_per_step_second_pass": round(ms_serial, 4),
        "kernel_table": "second pass of the same steps: a context with SYMI_CTX_TIMING | SYMI_CTX_NO_OVERLAP",
        "launch": "HIP graph replay" if args.graph else "host launches",
        "nonempty_slots_mean": round(mean_nonempty, 2),
        "classes_with_tokens_mean": round(mean_active, 2),
        "kernels": kernels,
    }
    del st, inputs
    torch.cuda.empty_cache()
    return out


def summary(out):
    """The few figures of another workload that ride along on the main line."""
    ks = out["kernels"]
    gemm = {n: e["TFLOP/s"] for n, e in ks.items() if n.startswith("gemm_") and "TFLOP/s" in e}
    peak = MFMA_BF16_PEAK_TF if out["dtype"] == "bf16" else FP32_VEC_PEAK_TF
    s = {"ms_per_step": out["ms_per_step"], "tokens_per_s": out["value"], "steps": out["steps"],
         "fwd_bwd_tokens_per_s": out["fwd_bwd_tokens_per_s"]}
    if "adam_to_replicas" in ks:
        s["adam_GB/s"] = ks["adam_to_replicas"]["GB/s"]
        s["adam_frac_of_hbm"] = round(ks["adam_to_replicas"]["GB/s"] / HBM_PEAK_GBS, 4)
    if gemm:
        s["gemm_TFLOP/s"] = gemm
        s["gemm_frac_of_peak_min_max"] = [round(min(gemm.values()) / peak, 4), round(max(gemm.values()) / peak, 4)]
    for n in ("gather_rows", "combine", "dispatch_bwd", "route"):
        if n in ks and "GB/s" in ks[n]:
            s[n + "_GB/s"] = ks[n]["GB/s"]
    return s


def cpu_baseline(c):
    """The oracle as it stands, timed on a bounded sample of the same workload: whole
    iterations on the first Ts tokens (all classes, full widths), Ts chosen so that one
    sampled iteration is at most 0.75 TFLOP of fp64 work."""
    import numpy as np
    import torch
    import workloads as wl
    from oracle import symi_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1

    per_token = 18.0 * c.k * c.d * c.f
    Ts = c.T
    while Ts > 256 and Ts * per_token > 0.75e12:
        Ts //= 2
    Es = min(c.E, 64)                        # classes whose shard the sampled Adam step covers
    dev = "cuda" if torch.cuda.is_available() else "cpu"     # where the inputs are drawn, nothing else
    W1g, W2g = wl.make_class_weights(c, dev)
    W1 = np.empty(tuple(W1g.shape), np.float32)
    W2 = np.empty(tuple(W2g.shape), np.float32)
    for e in range(c.E):
        W1[e] = W1g[e].float().cpu().numpy()
        W2[e] = W2g[e].float().cpu().numpy()
    del W1g, W2g
    per = c.P_e // c.N
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0, step=1)
    n1 = 2 * c.f * c.d                        # partition 0 owns [0, per) of the flat vector [W1 | W2]
    flat = np.concatenate([W1[:Es].reshape(Es, -1)[:, :min(per, n1)],
                           W2[:Es].reshape(Es, -1)[:, :max(per - n1, 0)]], 1).copy()
    hist_prev = np.zeros(c.E, dtype=np.int64)
    t_layer = t_adam = 0.0
    n_it = 0
    stages = {}
    # whole iterations of the workload until about 10 s of oracle time are spent (at most 3)
    for it in range(min(max(c.iters, 1), 3)):
        Xt = wl.make_tokens(c, it, dev)
        X = Xt[:Ts].float().cpu().numpy()
        z = wl.make_logits(c, it, dev, tokens=Xt)[:Ts].cpu().numpy()
        dY = wl.make_upstream_grad(c, it, dev)[:Ts].float().cpu().numpy()
        del Xt
        def stage(name, fn):
            t0 = time.perf_counter()
            r = fn()
            dt = time.perf_counter() - t0
            stages[name] = stages.get(name, 0.0) + dt
            return r, dt
        (idx, gate, hist), d1 = stage("route", lambda: O.route(z, c.k, True))
        (counts, placement, first), d2 = stage("place", lambda: O.place(hist_prev, c.S_tot))
        _, d3 = stage("dispatch", lambda: O.dispatch(idx, counts, first))
        _, d4 = stage("layer_fwd", lambda: O.moe_forward(X, idx, gate, W1, W2))
        (dX, dW1, dW2, dgate), d5 = stage("layer_bwd", lambda: O.moe_backward(X, idx, gate, W1, W2, dY))
        _, d6 = stage("route_bwd", lambda: O.route_backward(z, idx, gate, dgate, True))
        (n_counts, n_place, n_first), d7 = stage("place_next", lambda: O.place(hist, c.S_tot))
        t_layer += d1 + d2 + d3 + d4 + d5 + d6 + d7
        sub_place = np.array([e for e in n_place if e < Es], dtype=np.int32)
        W1s = np.zeros((len(sub_place),) + W1.shape[1:], np.float32)
        W2s = np.zeros((len(sub_place),) + W2.shape[1:], np.float32)
        _, d8 = stage("adam_to_replicas", lambda: O.adam_to_replicas(
            dW1[:Es], dW2[:Es], flat, np.zeros_like(flat), np.zeros_like(flat), sub_place, c.N, 0, hp,
            c.dtype == "bf16", W1s, W2s))
        t_adam += d8
        del dX, dW1, dW2, W1s, W2s
        hist_prev = hist
        n_it += 1
        if t_layer + t_adam >= 10.0:
            break

    est_step = (t_layer * (c.T / Ts) + t_adam * (c.E / Es)) / n_it
    # the oracle's stages beside the GPU's: seconds per full step (sample scaled as above)
    scale = {"adam_to_replicas": c.E / Es, "place": 1.0, "place_next": 1.0}     # the others grow with the tokens
    per_stage = {k: round(v / n_it * scale.get(k, c.T / Ts), 4) for k, v in stages.items()}
    return {"value": round(c.T / est_step, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "stage_seconds_per_step": per_stage,
            "sample": f"{n_it} iteration(s): layer fwd+bwd+routing on the first {Ts} of {c.T} tokens "
                      f"({t_layer:.2f} s), Adam+replica write on {Es} of {c.E} classes' shard ({t_adam:.2f} s); "
                      f"scaled linearly to one full step ({est_step:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c5")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other four workloads that ride along on the line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep every kernel on one stream also in the timed region (SYMI_CTX_NO_OVERLAP)")
    ap.add_argument("--graph", action="store_true",
                    help="timed region replays the steps from captured HIP graphs instead of launching "
                         "every kernel from the host")
    ap.add_argument("--dense-grads", action="store_true",
                    help="symi_expert_bwd / symi_adam_to_replicas (zero gradients of classes without "
                         "tokens written and read back) instead of the *_active pair")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device copy (reference for the HBM traffic counters)")
    ap.add_argument("--ceiling", action="store_true",
                    help="run the microbenchmarks of what the part sustains (register-only MFMA, the "
                         "GEMM loop with and without its ingredients, the Adam stream mix, torch fill/"
                         "copy) instead of the benchmark; --steps = launches per figure")
    ap.add_argument("--extras", action="store_true",
                    help="time the router GEMM/backward and the per-slot replica gradient path on "
                         "--config instead of the benchmark")
    ap.add_argument("--survival", type=float, default=None, metavar="CAPACITY_FACTOR",
                    help="print the token survival per iteration of --config under this capacity "
                         "factor (adaptive vs. uniform placement) instead of the benchmark")
    args = ap.parse_args()
    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.survival is not None:
        survival(args)
        return
    if args.extras:
        extras(args)
        return
    if args.ceiling:
        ceilings(args)
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the path; --gpus must be 1 "
              "(no collectives are part of it)", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as wl
    torch.cuda.set_device(0)
    c = wl.get_config(args.config)
    out = measure(c, args, args.steps, args.warmup)
    if not args.no_other_configs:
        # the other workloads, briefly (each one whole cycle of its iterations at least)
        out["other_configs"] = {}
        for name in sorted(wl.CONFIGS):
            if name == c.name:
                continue
            o = wl.get_config(name)
            out["other_configs"][name] = summary(measure(o, args, max(20, o.iters), 5))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(c)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
