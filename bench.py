#!/usr/bin/env python3
"""Benchmark of the Pier optimizer hot path on one MI355X.

A "step" is one outer round of the whole path on one batch of synthetic input:
H inner AdamW launches for each of the G group replicas (pier_inner_adamw), then
one outer step (pier_outer_step) - at the GPT-2 XL configuration by default
(N = 1 557 611 200 fp32 parameters, G = 8, H = 100: 800 + 1 kernel launches per
step).  All state and one gradient buffer per replica are resident in HBM before
the timed region; the gradients are reused by every inner step (their values do not
change the kernels' work).  Prints ONE JSON line.

`value` = parameters updated per second = N * (G*H + 1) / seconds per step, where an
inner launch updates the N parameters of one replica and the outer step the N
parameter positions of the synchronised model.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E peak

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the
# same counters' reading of a plain copy kernel); summary in
# profiles/kernels_gpt2_xl_hbm_traffic_pmc.md.  Only valid for the workload it was taken on.
MEASURED_TRAFFIC_GB = {"gpt2_xl": {"adamw": 44.003, "outer": 125.006, "lazy_start": 31.543}}
TRAFFIC_NOTE = ("GB per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script "
                "(profiles/kernels_gpt2_xl_hbm_traffic_pmc.md); a constant, not measured by this run")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="gpt2_xl")
    ap.add_argument("--inner-steps", type=int, default=0, help="override H (inner steps per round)")
    ap.add_argument("--no-offload", action="store_true", help="skip the host-offload measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-arena", action="store_true", help="plain allocations instead of the probed arena")
    ap.add_argument("--no-plain", action="store_true",
                    help="skip the closing measurement of the same kernels on plain allocations")
    ap.add_argument("--chunk-mib", type=int, default=0,
                    help="offload piece size; 0 = 256 MiB, or a sixteenth of one array (in steps of "
                         "16 MiB) when that is smaller, so that small models still fill the pipeline")
    ap.add_argument("--offload-slots", type=int, default=0,
                    help="staging slots of the offload stream (0: 3, or 20 when the outer state lives on the host)")
    ap.add_argument("--no-trailing", action="store_true",
                    help="host-offload workloads: make the compute stream wait for the copy-back")
    ap.add_argument("--variants", action="store_true",
                    help="also time the clipped step and the bf16-working-copy kernels")
    return ap.parse_args()


def _oracle_rounds(args):
    """Worker: rounds of the oracle on a private slice for about budget_s seconds."""
    name, n, H, budget_s, seed = args
    import numpy as np
    from oracle import pier_oracle as O
    from pier_inputs import shapes
    w = shapes.workloads()[name]
    G = w.G
    rng = np.random.default_rng(seed)
    P = [rng.normal(0, w.param_std, n).astype(np.float32) for _ in range(G)]
    M = [np.zeros(n, np.float32) for _ in range(G)]
    V = [np.zeros(n, np.float32) for _ in range(G)]
    Gr = [rng.normal(0, w.grad_std, n).astype(np.float32) for _ in range(G)]
    a, Mo = P[0].copy(), np.zeros(n, np.float32)
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    lr_o, mu = w.fixed_outer or (1.1, 0.9)
    O.adamw(P[0], M[0], V[0], Gr[0], step=1, **hp)          # warm the library / page in
    t0 = time.perf_counter()
    rounds, t = 0, 1
    while True:
        for _ in range(H):
            t += 1
            for g in range(G):
                O.adamw(P[g], M[g], V[g], Gr[g], step=t, **hp)
        O.outer(P, a, Mo, mu=mu, lr=lr_o, phase=O.PIER)
        rounds += 1
        dt = time.perf_counter() - t0
        if dt > budget_s:
            return rounds, dt


def cpu_baseline(w):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: a slice of the flat
    parameter space, G replicas, a few inner steps and one outer step per round.  The oracle is
    single-threaded, so the headline figure is one core; `all_cores` runs the same loop in one
    process per core of this box's share on disjoint slices (the work is elementwise).  Runs
    before the GPU is touched, so the workers are plain forks."""
    import multiprocessing as mp
    from oracle import pier_oracle as O
    O.build()
    n, G, H = 1 << 22, w.G, 4
    rounds, dt = _oracle_rounds((w.name, n, H, 10.0, 0))
    out = {"value": rounds * n * (G * H + 1) / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
           "sample": "%d rounds of (G=%d x H=%d AdamW steps + 1 outer step) on a %d-element slice, "
                     "single-threaded C oracle, %.1f s" % (rounds, G, H, n, dt)}
    cores = max(1, min(16, os.cpu_count() or 1))
    if cores > 1:
        with mp.get_context("fork").Pool(cores) as pool:
            res = pool.map(_oracle_rounds, [(w.name, n, H, 6.0, k + 1) for k in range(cores)])
        out["all_cores"] = {"value": sum(r * n * (G * H + 1) / d for r, d in res), "unit": "params/s",
                            "cores": cores, "sample": "the same loop in %d processes, disjoint slices" % cores}
    return out


class State:
    """All buffers of the workload on the GPU (placed through the library's plan when an arena is
    given), initialised, and a context bound to them."""

    def __init__(self, w, arena, host_outer, stream):
        import torch
        import paper_2511_17849_amd as pier
        from pier_inputs import device as dev
        self.w, self.stream, self.host_outer = w, stream, host_outer
        G, numels = w.G, w.numels
        gdt = torch.bfloat16 if w.grad_bf16 else torch.float32
        # the 7B configuration keeps one gradient buffer for all replicas (each launch reads it whole,
        # so the traffic is the same): nine of its 26 GiB buffers fit the three address classes, and
        # only with a single gradient buffer do every replica's four streams lie in two classes
        B = pier.ModelBuffers(w.N, G, grad_dtype=gdt, arena=arena, outer_on_device=not host_outer,
                              shared_grad=host_outer)
        wrap = lambda ts, cs: [dev.FlatList.wrap(t, numels, c) for t, c in zip(ts, cs)]
        self.P, self.M1 = wrap(B.theta, B.classes["theta"]), wrap(B.m, B.classes["m"])
        self.V, self.Gd = wrap(B.v, B.classes["v"]), wrap(B.grad, B.classes["grad"])
        if host_outer:
            self.A = dev.FlatList(numels, pinned=True, zero=False)
            self.Mo = dev.FlatList(numels, pinned=True, zero=False)
        else:
            self.A = dev.FlatList.wrap(B.anchor, numels, B.classes["anchor"])
            self.Mo = dev.FlatList.wrap(B.momentum, numels, B.classes["momentum"])
        with torch.cuda.stream(stream):
            for fl in self.M1 + self.V:
                fl.flat.zero_()
            dev.init_params(self.P[0], w)
            for g in range(1, G):
                self.P[g].flat.copy_(self.P[0].flat)
            for g in range(1 if host_outer else G):
                self.Gd[g].fill_normal(seed=w.seed, stream=g, step=1, std=w.grad_std, hip_stream=stream)
        stream.synchronize()
        self.A.flat.copy_(self.P[0].flat)
        self.Mo.flat.zero_()
        torch.cuda.synchronize()
        self.ctx = pier.pier_ctx_create(numels, G)
        for g in range(G):
            pier.pier_bind_replica(self.ctx, g, self.P[g].tensors, self.M1[g].tensors, self.V[g].tensors,
                                   self.Gd[g].tensors, w.grad_bf16)
        if host_outer:
            pier.pier_bind_outer(self.ctx, pier.PIER_LOC_HOST_PINNED, self.A.flat, self.Mo.flat)
        else:
            pier.pier_bind_outer(self.ctx, pier.PIER_LOC_DEVICE, self.A.tensors, self.Mo.tensors)
        self.t = 0

    def inner_round(self, H, hp):
        import paper_2511_17849_amd as pier
        for _ in range(H):
            self.t += 1
            for g in range(self.w.G):
                pier.pier_inner_adamw(self.ctx, g, step=self.t, stream=self.stream, **hp)


def run_placed(args, w):
    """The timed rounds (and the variants and the offload stream) on placed buffers; returns the
    result record and whether an arena was used.  Everything it allocated is released on return."""
    import torch
    import paper_2511_17849_amd as pier
    from pier_inputs import device as dev
    N, G = w.N, w.G
    H = args.inner_steps or w.H
    K, W = args.steps, args.warmup
    bf16 = w.grad_bf16
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    lr_o, mu = w.fixed_outer or (1.1, 0.9)
    stream = torch.cuda.Stream()

    if args.chunk_mib <= 0:
        args.chunk_mib = min(256, max(16, -(-(4 * N // 16) // (16 << 20)) * 16))
    chunk = args.chunk_mib << 20
    # a workload whose outer step IS the offload stream runs it with trailing write-back: the next
    # round's inner steps start as soon as the last piece's kernel is done, the copy-back of the
    # last pieces overlaps them; that needs staging for the backlog the slower copy-back builds up
    offload_slots = args.offload_slots or (20 if w.offload else 3)

    # HBM layout: one arena over (almost) all free HBM is probed for its address classes and
    # the buffers one launch streams together are carved from different classes; if the
    # arena cannot be had, buffers are allocated kind by kind instead
    arena, placement = None, "separate allocations, kind by kind"
    if not args.no_arena:
        try:
            free, _ = torch.cuda.mem_get_info()
            arena = pier.HbmArena(free - (8 << 30) - (offload_slots * 2 * chunk if w.offload else 0), stream=stream)
            placement = "probed arena of %d GiB, %d address classes, buffers placed by pier_placement_plan" % (
                arena.buf.numel() >> 30, arena.n_classes)
            print("bench.py: %s; class map %s" % (placement, "".join(str(c) for c in arena.classes)), file=sys.stderr)
        except (MemoryError, RuntimeError, pier.PierError) as e:
            print("bench.py: no arena (%s); allocating kind by kind" % e, file=sys.stderr)
    # workloads whose outer state lives in pinned host memory (the 7B configuration) take the
    # offload stream as their outer step; the PCIe time is then part of the step and `value`
    # is flagged as PCIe-inclusive in config
    host_outer = w.offload
    try:
        S = State(w, arena, host_outer, stream)
    except (MemoryError, pier.PierError) as e:
        if arena is None:
            raise
        # the probed classes leave no room for this model's plan: run on plain allocations instead
        print("bench.py: the placement plan does not fit the probed arena (%s); allocating kind by kind" % e,
              file=sys.stderr)
        arena, placement = None, "separate allocations, kind by kind (the plan did not fit the probed arena)"
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        S = State(w, None, host_outer, stream)
    ctx = S.ctx
    if host_outer:
        ws = torch.empty(2 * chunk * offload_slots, dtype=torch.uint8, device="cuda")
        s_in, s_out = torch.cuda.Stream(), torch.cuda.Stream()
        pier.pier_ctx_set_offload_writeback(ctx, 0 if args.no_trailing else 1)

    def outer_step():
        if host_outer:
            pier.pier_offload_stream(ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_PIER, chunk_bytes=chunk,
                                     workspace=ws, compute_stream=stream, h2d_stream=s_in, d2h_stream=s_out)
        else:
            pier.pier_outer_step(ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_PIER, stream=stream)

    def one_round(ev=None):
        if ev:
            ev[0].record(stream)
        S.inner_round(H, hp)
        if ev:
            ev[1].record(stream)
        outer_step()
        if ev:
            ev[2].record(stream)

    for _ in range(W):
        one_round()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        one_round(evs[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    inner_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / (K * G * H)     # per AdamW launch
    outer_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / K               # per outer launch

    def timed(fn, n):
        """Average milliseconds of n calls of fn after one untimed call."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # after the timed region: 20 more outer steps timed one by one (a round has only one)
    outer_each = []
    if not host_outer:
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for e0, e1 in pairs:
            e0.record(stream)
            outer_step()
            e1.record(stream)
        torch.cuda.synchronize()
        outer_each = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)
    gbytes = 26 if bf16 else 28
    inner_gbps = gbytes * N / inner_ms / 1e6
    outer_bpe = 8 * G + 16
    outer_gbps = outer_bpe * N / outer_ms / 1e6
    traffic = MEASURED_TRAFFIC_GB.get(w.name, {})
    ms_per_step = dt / K * 1e3
    value = N * (G * H + 1) / (dt / K)

    out = {
        "metric": "params updated/sec, inner AdamW (G x H launches) + outer Pier step, 1 GPU",
        "value": value, "unit": "params/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "f32 (bf16 gradients)", "data": "synthetic",
        "config": {"workload": "%s: N=%d fp32 params in %d tensors, G=%d replicas, H=%d inner steps per "
                               "round, %s outer step (mu=%.2f, outer lr=%.2f)" %
                               (w.name, N, len(w.numels), G, H,
                                "host-offload (PCIe-inclusive, %d MiB pieces, %d staging slots, %s write-back)" %
                                (args.chunk_mib, offload_slots, "blocking" if args.no_trailing else "trailing")
                                if host_outer
                                else "resident", mu, lr_o),
                   "hbm_placement": placement},
        # the paper publishes no figure for this path (hence vs_baseline null); its own numbers are
        # whole-training runtime ratios on other machines
        "paper_context": "end-to-end training speedups over AdamW data parallelism, GPT-2 XL: 2.7-3.7x on "
                         "256 A100 (Perlmutter), 1.2-1.9x on 64-128 GH200 (Vista); none for the optimizer step",
        "roofline": {"bound": "hbm", "kernel": "adamw_kernel (pier_inner_adamw)", "achieved": inner_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": inner_gbps / HBM_PEAK_GBPS,
                     "traffic": traffic.get("adamw"), "traffic_unit": TRAFFIC_NOTE,
                     "algorithmic_GB_per_launch": gbytes * N / 1e9,
                     "bytes_per_param": gbytes, "avg_launch_ms": inner_ms,
                     "launches_timed": K * G * H},
        "roofline_outer": {"bound": "pcie (host-offload stream; achieved = HBM bytes of the kernels over the "
                                    "PCIe-bound wall time)" if host_outer else "hbm",
                           "kernel": "outer_kernel (pier_offload_stream)" if host_outer else
                                     "outer_kernel (pier_outer_step, Pier phase)",
                           "achieved": outer_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                           "frac": outer_gbps / HBM_PEAK_GBPS, "traffic": traffic.get("outer"),
                           "traffic_unit": TRAFFIC_NOTE,
                           "algorithmic_GB_per_launch": outer_bpe * N / 1e9,
                           "bytes_per_param": outer_bpe, "avg_launch_ms": outer_ms, "launches_timed": K},
    }
    if outer_each:
        out["roofline_outer"].update({"median_launch_ms_of_20_more": outer_each[len(outer_each) // 2],
                                      "min_max_launch_ms_of_20_more": [outer_each[0], outer_each[-1]]})
    if not host_outer:
        # the lazy-start synchronisation (Algorithm 1): theta_0, anchor, M read; anchor, M written
        ms = timed(lambda: pier.pier_outer_step(ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_WARMUP,
                                                stream=stream), 20)
        out["roofline_lazy_start"] = {"bound": "hbm", "kernel": "lazy_start_kernel (pier_outer_step, lazy-start phase)",
                                      "achieved": 20 * N / ms / 1e6, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                      "frac": 20 * N / ms / 1e6 / HBM_PEAK_GBPS, "bytes_per_param": 20,
                                      "traffic": traffic.get("lazy_start"), "traffic_unit": TRAFFIC_NOTE,
                                      "algorithmic_GB_per_launch": 20 * N / 1e9,
                                      "avg_launch_ms": ms, "launches_timed": 20}

    if args.variants and not host_outer:
        P = S.P
        n_var = 20

        def all_replicas(call):
            def f():
                S.t += 1
                for g in range(G):
                    call(g)
            return f

        var = {}
        ms = timed(all_replicas(lambda g: pier.pier_inner_adamw_clipped(ctx, g, step=S.t, max_norm=1.0,
                                                                       stream=stream, **hp)), n_var) / G
        var["adamw_clipped"] = {"ms": ms, "bytes_per_param": gbytes + (2 if bf16 else 4),
                                "GBps": (gbytes + (2 if bf16 else 4)) * N / ms / 1e6, "launches": n_var * G}
        Wb = []
        try:
            for g in range(G):
                flat = arena.alloc(N, torch.bfloat16, P[g].cls)[0] if arena is not None else \
                    torch.empty(N, dtype=torch.bfloat16, device="cuda")
                Wb.append([flat[s0:s0 + n] for s0, n in zip(P[g].starts, w.numels)])
        except (MemoryError, RuntimeError) as e:
            print("bench.py: no room for the bf16 working copies (%s); those variants are skipped" % e, file=sys.stderr)
            Wb = []
        for g in range(len(Wb)):
            pier.pier_bind_shadow(ctx, g, Wb[g])
        if Wb:
            ms = timed(all_replicas(lambda g: pier.pier_inner_adamw(ctx, g, step=S.t, stream=stream, **hp)), n_var) / G
            var["adamw_bf16_working_copy"] = {"ms": ms, "bytes_per_param": gbytes + 2, "GBps": (gbytes + 2) * N / ms / 1e6,
                                              "launches": n_var * G}
            ms = timed(lambda: pier.pier_outer_step(ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_PIER,
                                                    stream=stream), n_var)
            var["outer_bf16_working_copy"] = {"ms": ms, "bytes_per_param": outer_bpe + 2 * G,
                                              "GBps": (outer_bpe + 2 * G) * N / ms / 1e6, "launches": n_var}
            for g in range(G):
                pier.pier_bind_shadow(ctx, g, None)
        del Wb
        out["variants"] = var

    if not args.no_offload:
        # the same outer step with anchor and M streamed from pinned host memory
        if not host_outer:
            hA, hM = dev.pinned_empty(N), dev.pinned_empty(N)      # exact size: pinned memory is scarce
            hM.zero_()
            hA.copy_(S.A.flat)
            pier.pier_bind_outer(ctx, pier.PIER_LOC_HOST_PINNED, hA, hM)
            ws = torch.empty(pier.pier_offload_workspace_bytes(ctx, chunk), dtype=torch.uint8, device="cuda")
            s_in, s_out = torch.cuda.Stream(), torch.cuda.Stream()
        pier.pier_ctx_set_offload_writeback(ctx, 0)
        best = None
        for _ in range(3):
            st = pier.pier_offload_stream(ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_PIER,
                                          chunk_bytes=chunk, workspace=ws, compute_stream=stream,
                                          h2d_stream=s_in, d2h_stream=s_out, want_stats=True)
            if best is None or st.wall_ms < best.wall_ms:
                best = st
        out["offload"] = {
            "entry": "pier_offload_stream", "chunk_mib": args.chunk_mib, "pieces": best.n_pieces,
            "slots": best.n_slots, "wall_ms": best.wall_ms,
            "h2d_GBps": best.h2d_bytes / best.h2d_ms / 1e6, "d2h_GBps": best.d2h_bytes / best.d2h_ms / 1e6,
            "pcie_GBps_each_way_over_wall": best.h2d_bytes / best.wall_ms / 1e6,
            "kernel_ms": best.kernel_ms, "first_reload_to_last_kernel_ms": best.compute_ms,
            "overlap": max(best.h2d_ms, best.d2h_ms, best.kernel_ms) / best.wall_ms,
            "params_per_s": N / best.wall_ms * 1e3,
        }

    if not host_outer and G >= 3:
        # What the machine gives a PLAIN copy and a plain fill of model-sized buffers, by the array
        # library's own kernels, in the same placement: the yardstick for mixed read/write streaming
        # (the state is no longer needed, so the replicas serve as scratch).  theta_0 and theta_2 share
        # an address class, theta_1 lies in the other one.
        ref = {}
        for name, fn, nbytes in (
                ("copy_across_classes", lambda: S.P[1].flat.copy_(S.P[0].flat), 8 * N),
                ("copy_within_a_class", lambda: S.P[2].flat.copy_(S.P[0].flat), 8 * N),
                ("fill", lambda: S.P[1].flat.zero_(), 4 * N)):
            with torch.cuda.stream(stream):
                ms = timed(fn, 20)
            ref[name] = {"GBps": nbytes / ms / 1e6, "frac": nbytes / ms / 1e6 / HBM_PEAK_GBPS, "ms": ms}
        ref["what"] = ("torch copy_ / zero_ of one %d-byte buffer, 20 launches each: what plain library kernels "
                       "stream at on this GPU" % (4 * N))
        if arena is not None:
            # and the best the placement probe saw at set-up: two 2 GiB buffers streamed in place with
            # trivial arithmetic (read both, add, write both) - the two kernels' access pattern at its simplest
            ref["probe_best_two_buffer_in_place"] = {"GBps": 1e3 * arena.probe["best_rate"],
                                                     "frac": 1e3 * arena.probe["best_rate"] / HBM_PEAK_GBPS,
                                                     "cross_class_threshold_GBps": 1e3 * arena.probe["threshold"],
                                                     "pairs_timed": arena.probe["n_pairs"]}
        out["hbm_reference"] = ref
    pier.pier_ctx_destroy(ctx)
    return out, arena is not None


def run_plain(args, w, out):
    """What a caller gets WITHOUT the probe and the plan: the same kernels on plain allocations
    made kind by kind, a few launches."""
    import torch
    import paper_2511_17849_amd as pier
    N, G = w.N, w.G
    H = args.inner_steps or w.H
    bf16 = w.grad_bf16
    gbytes, outer_bpe = (26 if bf16 else 28), 8 * G + 16
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    lr_o, mu = w.fixed_outer or (1.1, 0.9)
    stream = torch.cuda.Stream()
    S2 = State(w, None, False, stream)
    Hp = min(H, 5)
    S2.inner_round(1, hp)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(stream)
    S2.inner_round(Hp, hp)
    ev[1].record(stream)
    for _ in range(10):
        pier.pier_outer_step(S2.ctx, outer_lr=lr_o, mu=mu, phase=pier.PIER_PHASE_PIER, stream=stream)
    ev[2].record(stream)
    torch.cuda.synchronize()
    p_inner = ev[0].elapsed_time(ev[1]) / (Hp * G)
    p_outer = ev[1].elapsed_time(ev[2]) / 10
    out["roofline_plain_allocations"] = {
        "what": "the same kernels on plain device allocations made kind by kind (no probe, no placement plan)",
        "adamw": {"achieved": gbytes * N / p_inner / 1e6, "frac": gbytes * N / p_inner / 1e6 / HBM_PEAK_GBPS,
                  "avg_launch_ms": p_inner, "launches_timed": Hp * G},
        "outer": {"achieved": outer_bpe * N / p_outer / 1e6, "frac": outer_bpe * N / p_outer / 1e6 / HBM_PEAK_GBPS,
                  "avg_launch_ms": p_outer, "launches_timed": 10},
        "unit": "GB/s", "peak": HBM_PEAK_GBPS}
    pier.pier_ctx_destroy(S2.ctx)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
              "supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)
    from pier_inputs import shapes
    w = shapes.workloads()[args.workload]
    baseline = None
    if not args.no_cpu_baseline:
        baseline = cpu_baseline(w)      # before any GPU call
    import gc
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    out, had_arena = run_placed(args, w)
    if had_arena and not w.offload and not args.no_plain:
        gc.collect()                  # the arena held nearly all HBM: it is gone with run_placed's locals
        torch.cuda.empty_cache()
        run_plain(args, w, out)
    if baseline is not None:
        out["cpu_baseline"] = baseline
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
