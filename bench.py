#!/usr/bin/env python3
"""Benchmark of the R-Sparse linear layer on one MI355X.

Headline workload (benchmark configs[4], the largest single-GPU one at batch 1): the seven linears of one
Llama-3-70B decoder layer -- q, o 8192 x 8192; k, v 8192 -> 1024; gate, up 8192 -> 28672; down 28672 -> 8192 --
bf16, rank 1024, 50 % channel sparsity, one token.  One "step" = one pass of the hot path (threshold, compaction,
gather-GEMV, both low-rank products, sum, store) over all seven: four calls, as a decoder would issue them
(q / k / v grouped on the shared input, o, gate / up grouped, down), each call one launch of the hot-path kernel.
The same line carries configs[1] (Llama-2-7B MLP: gate / up 4096 -> 11008, down 11008 -> 4096, rank 512) and
configs[0] (4096 x 4096 fp16, rank 256 -- the shape the 1.6x target is anchored on) under "workloads", each with its
own roofline, dense baseline and speed-up.  Steps walk rings of distinct prepared layers (>= 1 GiB of weights per
ring) so that weight bytes come from HBM; inputs are resident before the timed region.  Both ways of issuing the
launches (plain stream launches, replay of a captured HIP graph) and both weight layouts of the library
(column-major with the column-tile kernel, strips with the strip kernel) are timed; the fastest is the value, and
the line says which it was.

Prints ONE JSON line.  `value` = microseconds per R-Sparse linear of the headline workload.  `roofline` is for
the kernel the calls run: the bytes the method must move per launch over the launch's event-timed duration;
`cpu_baseline` is the fp64 CPU oracle on the host cores on a bounded sample.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
REPEATS = 10               # timed brackets of `steps` steps each; the median is reported
K_TOKENS = 32              # tokens per linear for the statistics of k (kept channels)
STRIP_COLS = 128           # strip width of the strip-layout variant
CHANNEL_MAJOR_MIN_WEIGHTS = 1 << 26   # column layout: calls that read this many weights keep S_r V_r^T channel-major as well


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def shape_batch_sweep(args, torch, np, rs, synth):
    """Other configs' shapes and batch sizes: us per linear for R-Sparse and for the dense baseline, each
    over a ring of distinct layers (>= 0.9 GiB of weights), HIP-graph replay, 50 % per-token sparsity."""
    cases = [  # (label, d_in, d_out, rank, dtype, input kind, batches)
        ("c0 4096x4096 f16 r256", 4096, 4096, 256, synth.F16, "dmodel", (1,)),
        ("c2 q/k/v/o 4096x4096 bf16 r256", 4096, 4096, 256, synth.BF16, "dmodel", (1, 2, 4, 8)),
        ("c3 gate/up 4096x14336 bf16 r256", 4096, 14336, 256, synth.BF16, "dmodel", (1, 4, 16)),
        ("c3 k/v 4096x1024 bf16 r128", 4096, 1024, 128, synth.BF16, "dmodel", (1, 16)),
        ("c4 q/o 8192x8192 bf16 r1024", 8192, 8192, 1024, synth.BF16, "dmodel", (1, 8, 32)),
        ("c4 gate/up 8192x28672 bf16 r1024", 8192, 28672, 1024, synth.BF16, "dmodel", (1, 8, 32)),
        ("c4 down 28672x8192 bf16 r1024", 28672, 8192, 1024, synth.BF16, "down", (1, 32)),
    ]
    stream = torch.cuda.current_stream()
    out = []
    for label, d_in, d_out, rank, dt, kind, batches in cases:
        n_ring = max(2, min(32, int(0.9 * 2 ** 30 / (d_in * d_out * 2)) + 1))
        L = synth.random_layer(d_in, d_out, rank, dt, seed=d_in + d_out)
        src = (synth.DModelInput if kind == "dmodel" else synth.DownInput)(d_in, config=5, linear=0)
        tau = rs.rsparse_calibrate_tau(synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), dt), dt, 0.5)
        maxb = max(batches)
        layers = []
        for i in range(n_ring):
            cfg = rs.make_config(d_in, d_out, rank, tau, dt, max_batch=maxb, dense_rowmajor=1, lowrank_channel_major=1)
            layers.append(rs.rsparse_prepare_factors(cfg, L.W16, L.U16, L.SV16))
        for B in batches:
            xs = [torch.from_numpy(synth.encode16(src.tokens(B, offset=10 + i), dt).view(np.int16)).cuda()
                  for i in range(n_ring)]
            ys = [torch.zeros((B, d_out), dtype=torch.int16, device="cuda") for _ in range(n_ring)]

            def run(fn):
                def one_pass(sptr):
                    for layer, x, y in zip(layers, xs, ys):
                        fn(layer, x.data_ptr(), B, y.data_ptr(), sptr)
                one_pass(stream.cuda_stream)
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    one_pass(torch.cuda.current_stream().cuda_stream)
                for _ in range(3):
                    g.replay()
                torch.cuda.synchronize()
                reps = max(3, int(2000 / n_ring / max(1.0, d_in * d_out / 4096 / 4096)))
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    g.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) * 1000.0 / (reps * n_ring)

            us_rs = run(rs.rsparse_linear)
            k_union = len(rs.rsparse_last_active(layers[-1], -1))
            us_dense = run(rs.rsparse_dense_ref)
            req = rs.rsparse_required_bytes(layers[0], B, k_union)
            est_rs, est_dense, use = rs.rsparse_plan_layer(d_in, d_out, rank, 0.5, 1, B)
            out.append({"case": label, "batch": B, "ring_layers": n_ring, "k_union": k_union,
                        "us_rsparse": round(us_rs, 2), "us_dense": round(us_dense, 2),
                        "speedup": round(us_dense / us_rs, 3),
                        "plan": "rsparse" if use else "dense", "us_as_planned": round(us_rs if use else us_dense, 2),
                        "plan_estimates_us": [round(est_rs, 1), round(est_dense, 1)], "required_MB": round(req / 1e6, 2),
                        "gbs_required": round(req / us_rs / 1e3, 1), "frac_of_8TBs": round(req / us_rs / 8e6, 3),
                        "dense_gbs": round(rs.rsparse_dense_bytes(layers[0], B) / us_dense / 1e3, 1)})
            log(str(out[-1]))
        for layer in layers:
            layer.destroy()
        torch.cuda.empty_cache()
    return out


def decoder_layer_sweep(torch, np, rs, synth):
    """configs[2]: the seven linears of one Llama-2-7B decoder layer (q, k, v, o 4096x4096; gate, up
    4096->11008; down 11008->4096), bf16, 50 % sparsity, rank d_model / 16 = 256, batch 1, 2, 4, 8.
    Four calls per layer: q/k/v grouped, o, gate/up grouped, down.  Ring of 3 layers (1.2 GiB)."""
    dt, r = synth.BF16, 256
    shapes = [("q", 4096, 4096, "dmodel"), ("k", 4096, 4096, "dmodel"), ("v", 4096, 4096, "dmodel"),
              ("o", 4096, 4096, "dmodel"), ("gate", 4096, 11008, "dmodel"), ("up", 4096, 11008, "dmodel"),
              ("down", 11008, 4096, "down")]
    n_ring, maxb = 3, 8
    stream = torch.cuda.current_stream()
    ring = []
    for blk in range(n_ring):
        blkl = {}
        for li, (name, d_in, d_out, kind) in enumerate(shapes):
            L = synth.random_layer(d_in, d_out, r, dt, seed=7000 + li)
            src = (synth.DModelInput if kind == "dmodel" else synth.DownInput)(d_in, config=2, linear=li)
            tau = rs.rsparse_calibrate_tau(synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), dt), dt, 0.5)
            cfg = rs.make_config(d_in, d_out, r, tau, dt, max_batch=maxb, dense_rowmajor=1, lowrank_channel_major=1)
            x = torch.from_numpy(synth.encode16(src.tokens(maxb, offset=20 + blk), dt).view(np.int16)).cuda()
            y = torch.zeros((maxb, d_out), dtype=torch.int16, device="cuda")
            blkl[name] = (rs.rsparse_prepare_factors(cfg, L.W16, L.U16, L.SV16), x, y)
        ring.append(blkl)
    out = []

    def one_layer(b, B, sptr, fn_group, fn_one):
        fn_group([b[n][0] for n in "qkv"], b["q"][1].data_ptr(), B, [b[n][2].data_ptr() for n in "qkv"], sptr)
        fn_one(b["o"][0], b["o"][1].data_ptr(), B, b["o"][2].data_ptr(), sptr)
        fn_group([b["gate"][0], b["up"][0]], b["gate"][1].data_ptr(), B, [b["gate"][2].data_ptr(), b["up"][2].data_ptr()], sptr)
        fn_one(b["down"][0], b["down"][1].data_ptr(), B, b["down"][2].data_ptr(), sptr)

    def timed(B, fn_group, fn_one, reps=60, layer_fn=None):
        def one_pass(sptr):
            for b in ring:
                (layer_fn or one_layer)(b, B, sptr, fn_group, fn_one)
        one_pass(stream.cuda_stream)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one_pass(torch.cuda.current_stream().cuda_stream)
        for _ in range(20):
            g.replay()
        torch.cuda.synchronize()
        best = 1e30
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                g.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1000.0 / (reps * n_ring))
        return best

    def set_all(**kw):
        for b in ring:
            for layer, _, _ in b.values():
                rs.rsparse_set_tuning(layer, **kw)

    for B in (1, 2, 4, 8):
        row = {"case": "c2 decoder layer (7 linears, 4 calls) bf16 r256", "batch": B}
        set_all(launches=1)
        row["us_rsparse_one_launch"] = round(timed(B, rs.rsparse_linear_group, rs.rsparse_linear), 2)
        set_all(launches=2)
        row["us_rsparse_two_launches"] = round(timed(B, rs.rsparse_linear_group, rs.rsparse_linear), 2)
        set_all()
        row["us_dense"] = round(timed(B, rs.rsparse_dense_ref_group, rs.rsparse_dense_ref), 2)
        row["speedup"] = round(row["us_dense"] / min(row["us_rsparse_one_launch"], row["us_rsparse_two_launches"]), 3)
        # per call, what rsparse_plan_layer picks at this batch (byte model + fixed launch costs): R-Sparse or dense
        plan = {"qkv": rs.rsparse_plan_layer(4096, 4096, r, 0.5, 3, B)[2], "o": rs.rsparse_plan_layer(4096, 4096, r, 0.5, 1, B)[2],
                "gate_up": rs.rsparse_plan_layer(4096, 11008, r, 0.5, 2, B)[2], "down": rs.rsparse_plan_layer(11008, 4096, r, 0.5, 1, B)[2]}

        def planned_layer(b, Bn, sptr, _g, _o):
            grp = lambda use: rs.rsparse_linear_group if use else rs.rsparse_dense_ref_group
            one = lambda use: rs.rsparse_linear if use else rs.rsparse_dense_ref
            grp(plan["qkv"])([b[n][0] for n in "qkv"], b["q"][1].data_ptr(), Bn, [b[n][2].data_ptr() for n in "qkv"], sptr)
            one(plan["o"])(b["o"][0], b["o"][1].data_ptr(), Bn, b["o"][2].data_ptr(), sptr)
            grp(plan["gate_up"])([b["gate"][0], b["up"][0]], b["gate"][1].data_ptr(), Bn,
                                 [b["gate"][2].data_ptr(), b["up"][2].data_ptr()], sptr)
            one(plan["down"])(b["down"][0], b["down"][1].data_ptr(), Bn, b["down"][2].data_ptr(), sptr)

        set_all(launches=1)
        row["plan"] = {k: ("rsparse" if v else "dense") for k, v in plan.items()}
        row["us_planned"] = round(timed(B, None, None, layer_fn=planned_layer), 2)
        row["speedup_planned"] = round(row["us_dense"] / row["us_planned"], 3)
        set_all()
        out.append(row)
        log(str(row))
    for b in ring:
        for layer, _, _ in b.values():
            layer.destroy()
    torch.cuda.empty_cache()
    return out


def workloads(synth):
    return {
        "configs[4]": dict(
            title="configs[4]: Llama-3-70B decoder-layer shapes, bf16, batch 1, rank 1024, 50 % channel sparsity; "
                  "step = the 7 linears of one layer in 4 calls (q/k/v grouped, o, gate/up grouped, down)",
            dtype=synth.BF16, rank=1024, blocks=1,
            linears=[("q", 8192, 8192, "dmodel"), ("k", 8192, 1024, "dmodel"), ("v", 8192, 1024, "dmodel"),
                     ("o", 8192, 8192, "dmodel"), ("gate", 8192, 28672, "dmodel"), ("up", 8192, 28672, "dmodel"),
                     ("down", 28672, 8192, "down")],
            calls=[["q", "k", "v"], ["o"], ["gate", "up"], ["down"]]),
        "configs[1]": dict(
            title="configs[1]: Llama-2-7B MLP, bf16, batch 1, rank 512, 50 % channel sparsity; step = gate/up "
                  "(4096 -> 11008, grouped) + down (11008 -> 4096)",
            dtype=synth.BF16, rank=512, blocks=4,
            linears=[("gate", 4096, 11008, "dmodel"), ("up", 4096, 11008, "dmodel"), ("down", 11008, 4096, "down")],
            calls=[["gate", "up"], ["down"]]),
        "configs[0]": dict(
            title="configs[0]: one linear 4096 x 4096, fp16, batch 1, rank 256, 50 % channel sparsity",
            dtype=synth.F16, rank=256, blocks=32,
            linears=[("lin", 4096, 4096, "dmodel")],
            calls=[["lin"]]),
    }


class Ring:
    """`blocks` copies of a workload's linears at distinct device addresses (one layout), tokens and outputs."""

    def __init__(self, wl, cfg_no, sparsity, strip_cols, rs, synth, torch, np, base=None, rank=None, rowmajor=1):
        self.wl, self.rs, self.torch = wl, rs, torch
        dt = wl["dtype"]
        rank = wl["rank"] if rank is None else rank
        self.base = base if base is not None else {}
        self.src, self.tau, self.blocks, self.channel_major = {}, {}, [], {}
        for li, (name, d_in, d_out, kind) in enumerate(wl["linears"]):
            if name not in self.base:
                # i.i.d. operands of the workload's scales: kernel time, traffic and parity do not depend on W being an
                # SVD product (the parity tests also run the exact U diag(sigma) V^T construction)
                self.base[name] = synth.random_layer(d_in, d_out, wl["rank"], dt, seed=1000 * cfg_no + 10 * li)
            src = (synth.DModelInput if kind == "dmodel" else synth.DownInput)(d_in, config=cfg_no, linear=li)
            self.src[name] = src
            calib = synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), dt)
            self.tau[name] = {s: rs.rsparse_calibrate_tau(calib, dt, s) for s in {0.4, 0.5, 0.7, sparsity}}
        for blk in range(wl["blocks"]):
            b, xs = {}, {}
            for call in wl["calls"]:
                first = next(l for l in wl["linears"] if l[0] == call[0])
                x16 = synth.encode16(self.src[first[0]].tokens(1, offset=1 + blk), dt)      # a call's linears share the token
                xd = torch.from_numpy(x16.view(np.int16)).cuda()
                for name in call:
                    _, d_in, d_out, _ = next(l for l in wl["linears"] if l[0] == name)
                    L = self.base[name]
                    # column layout: the layers of a call (one launch) that reads 2^26 weights or more also keep S_r V_r^T
                    # channel-major, so that stage 1 reads the dropped channels' rows only (measured to pay from that
                    # size on -- the launch is then long enough to hide that t is published later -- and to cost time below)
                    call_weights = sum(di * do for n2, di, do, _ in wl["linears"] if n2 in call)
                    cm = 1 if strip_cols == 0 and rank and call_weights >= CHANNEL_MAJOR_MIN_WEIGHTS else 0
                    self.channel_major[name] = cm
                    cfg = rs.make_config(d_in, d_out, rank, self.tau[name][sparsity], dt, max_batch=1,
                                         dense_rowmajor=rowmajor if strip_cols == 0 else 0, strip_cols=strip_cols,
                                         lowrank_channel_major=cm)
                    layer = rs.rsparse_prepare_factors(cfg, L.W16, L.U16[:, :rank] if rank else None,
                                                       L.SV16[:rank] if rank else None)
                    b[name] = (layer, xd, torch.zeros((1, d_out), dtype=torch.int16, device="cuda"), x16)
            self.blocks.append(b)
        torch.cuda.synchronize()

    def layers(self):
        return [e[0] for b in self.blocks for e in b.values()]

    def set_all(self, **kw):
        for layer in self.layers():
            self.rs.rsparse_set_tuning(layer, **kw)

    def set_tau(self, s):
        for b in self.blocks:
            for name, e in b.items():
                self.rs.rsparse_set_tau(e[0], self.tau[name][s])

    def pass_fn(self, dense=False, separate=False):
        rs, calls = self.rs, self.wl["calls"]
        one = rs.rsparse_dense_ref if dense else rs.rsparse_linear
        group = rs.rsparse_dense_ref_group if dense else rs.rsparse_linear_group

        def run(sptr):
            for b in self.blocks:
                for call in calls:
                    if len(call) == 1 or separate:
                        for name in call:
                            layer, xd, yd, _ = b[name]
                            one(layer, xd.data_ptr(), 1, yd.data_ptr(), sptr)
                    else:
                        es = [b[n] for n in call]
                        group([e[0] for e in es], es[0][1].data_ptr(), 1, [e[2].data_ptr() for e in es], sptr)
        return run

    def destroy(self):
        for layer in self.layers():
            layer.destroy()
        self.blocks = []
        self.torch.cuda.empty_cache()


def make_timer(torch, args):
    stream = torch.cuda.current_stream()

    def timed(pass_fn, blocks, eager):
        """ms per step (= one block of the ring) over exactly args.steps steps; median of REPEATS brackets."""
        graph = None
        if not eager:
            pass_fn(stream.cuda_stream)                 # make sure everything is loaded before capture
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                pass_fn(torch.cuda.current_stream().cuda_stream)
        steps = max(blocks, (args.steps + blocks - 1) // blocks * blocks)       # whole ring passes

        def run(n_steps):
            for _ in range(max(1, n_steps // blocks)):
                graph.replay() if graph is not None else pass_fn(stream.cuda_stream)

        run(args.warmup)
        torch.cuda.synchronize()
        # the card idles (and clocks down) while the host builds layers or runs the oracle: keep it busy for
        # ~0.2 s untimed, then time `steps` steps REPEATS times, each bracketed by a synchronize
        t_busy = time.time()
        while time.time() - t_busy < 0.2:
            run(blocks * 8)
            torch.cuda.synchronize()
        samples = []
        for _ in range(REPEATS):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            run(steps)
            e1.record(stream)
            torch.cuda.synchronize()
            samples.append(e0.elapsed_time(e1) / steps)
        samples.sort()
        return samples[len(samples) // 2]

    def best(pass_fn, blocks):
        modes = {"eager": timed(pass_fn, blocks, True)}
        if not args.eager:
            modes["graph"] = timed(pass_fn, blocks, False)
        m = min(modes, key=modes.get)
        return modes[m], m, modes

    return timed, best


def traffic_from_profiles(kernel, cfg_label):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc (FETCH_SIZE scaled + WRITE_SIZE), from the summary
    committed under profiles/ (a line `traffic_bytes_per_launch[<kernel>][<workload>] = <bytes>`); None if absent."""
    pat = re.compile(r"traffic_bytes_per_launch\[%s\]\[%s\]\s*=\s*([0-9.eE+]+)" % (re.escape(kernel), re.escape(cfg_label)))
    d = os.path.join(ROOT, "profiles")
    if not os.path.isdir(d):
        return None
    for f in sorted(os.listdir(d)):
        if f.endswith((".md", ".txt")):
            m = pat.search(open(os.path.join(d, f)).read())
            if m:
                return float(m.group(1))
    return None


def measure_workload(label, cfg_no, args, mods, timers, want_cpu):
    torch, np, rs, synth, oracle = mods
    timed, best = timers
    wl = workloads(synth)[label]
    dt, stream = wl["dtype"], torch.cuda.current_stream()
    n_lin, n_calls, blocks = len(wl["linears"]), len(wl["calls"]), wl["blocks"]
    t0 = time.time()
    col = Ring(wl, cfg_no, args.sparsity, 0, rs, synth, torch, np)
    strip = Ring(wl, cfg_no, args.sparsity, STRIP_COLS, rs, synth, torch, np, base=col.base)
    log(f"{label}: rings resident ({blocks} block(s) x {n_lin} linears, two layouts; {time.time() - t0:.1f}s)")

    # ---- parity sanity on the timed configuration (block 0, both layouts) and k over K_TOKENS tokens per linear
    for ring in (col, strip):
        ring.pass_fn()(stream.cuda_stream)
    torch.cuda.synchronize()
    k_stats, req_bytes, dense_bytes = {}, {}, {}
    for name, d_in, d_out, kind in wl["linears"]:
        L, tau = col.base[name], col.tau[name][args.sparsity]
        for ring in (col, strip):
            layer, xd, yd, x16 = ring.blocks[0][name]
            want = oracle.rsparse_linear(L.W16, L.U16, L.SV16, x16, dt, dt, tau, nthreads=16)
            got = synth.decode16(yd.cpu().numpy().view(np.uint16), dt)
            rel = np.linalg.norm(got - want["Y"]) / np.linalg.norm(want["Y"])
            assert np.array_equal(rs.rsparse_last_active(layer, 0), want["act"][0]), f"{label} {name}: kept list differs"
            assert rel <= 2e-3, f"{label} {name}: rel L2 {rel}"
        layer, xd, yd, _ = col.blocks[0][name]
        toks = synth.encode16(col.src[name].tokens(K_TOKENS, offset=50), dt)
        ks = []
        for i in range(K_TOKENS):
            xt = torch.from_numpy(toks[i:i + 1].view(np.int16)).cuda()
            rs.rsparse_linear(layer, xt.data_ptr(), 1, yd.data_ptr(), stream.cuda_stream)
            ks.append(len(rs.rsparse_last_active(layer, -1)))
        k_stats[name] = {"mean": round(float(np.mean(ks)), 1), "min": int(min(ks)), "max": int(max(ks))}
        # bytes of the timed tokens themselves (every block of the ring), per linear
        kk = [len(rs.rsparse_last_active(b[name][0], -1)) if bi == 0 else None for bi, b in enumerate(col.blocks)]
        req_bytes[name] = rs.rsparse_required_bytes(layer, 1, int(round(np.mean(ks))))
        dense_bytes[name] = rs.rsparse_dense_bytes(layer, 1)
        del kk
    # exact k of the timed tokens: one pass, then read back every layer of the ring
    col.pass_fn()(stream.cuda_stream)
    torch.cuda.synchronize()
    req_total, req_less = 0, 0
    for b in col.blocks:
        for name, (layer, *_rest) in b.items():
            k_b = len(rs.rsparse_last_active(layer, -1))
            req_total += rs.rsparse_required_bytes(layer, 1, k_b)
            # secondary denominator: a layer whose stage 1 reads only the dropped channels' rows of S_r V_r^T
            # requests rank * k fewer elements than the required bytes count
            req_less += 2 * wl["rank"] * k_b * col.channel_major[name]
    req_step = req_total / blocks                                   # algorithmic bytes of one step
    requested_step = (req_total - req_less) / blocks
    dense_step = sum(dense_bytes.values())
    log(f"{label}: parity ok on both layouts; k per linear over {K_TOKENS} tokens: {k_stats}")

    # ---- R-Sparse, both layouts, both launch modes
    res = {}
    for lay, ring, kern in (("column", col, "k_rsparse_fused"), ("strip", strip, "k_rsparse_strip")):
        ms, mode, modes = best(ring.pass_fn(), blocks)
        res[lay] = {"us_per_linear": round(ms * 1000.0 / n_lin, 3), "launch_mode": mode, "kernel": kern,
                    "us_per_linear_by_launch_mode": {k: round(v * 1000.0 / n_lin, 3) for k, v in modes.items()},
                    "ms_per_step": ms}
    if any(col.channel_major.values()) and not args.no_extras:
        col.set_all(lowrank_wgs=-1)                                 # the same ring with stage 1 over the row-major copy
        ms, mode, modes = best(col.pass_fn(), blocks)
        col.set_all()
        res["column_rowmajor_stage1"] = {"us_per_linear": round(ms * 1000.0 / n_lin, 3), "launch_mode": mode,
                                         "kernel": "k_rsparse_fused",
                                         "us_per_linear_by_launch_mode": {k: round(v * 1000.0 / n_lin, 3) for k, v in modes.items()},
                                         "ms_per_step": ms}
    lay = min(res, key=lambda k: res[k]["ms_per_step"])
    ms_step = res[lay]["ms_per_step"]
    us_linear = ms_step * 1000.0 / n_lin
    # ---- dense GEMV baselines: every dense kernel of the library, same grouping; the best is the baseline
    dense_us = {}
    for key, ring, kw in (("rowdot", col, dict(dense_kernel=2)), ("axpy", col, dict(dense_kernel=1)),
                          ("strip", strip, dict(dense_kernel=1))):
        ring.set_all(**kw)
        dense_us[key] = best(ring.pass_fn(dense=True), blocks)[0] * 1000.0 / n_lin
        ring.set_all()
    best_dense = min(dense_us.values())
    us_launch = ms_step * 1000.0 / n_calls
    bytes_launch = req_step / n_calls
    achieved = bytes_launch / (us_launch * 1e-6) / 1e9
    kern = res[lay]["kernel"]
    out = {
        "workload": wl["title"],
        "us_per_linear": round(us_linear, 3), "layout": lay, "launch_mode": res[lay]["launch_mode"],
        "ms_per_step": round(ms_step, 5), "linears_per_step": n_lin, "launches_per_step": n_calls,
        "by_layout": {k: {kk: vv for kk, vv in v.items() if kk != "ms_per_step"} for k, v in res.items()},
        "kept_channels": k_stats,
        "required_bytes_per_step": int(req_step), "dense_bytes_per_step": int(dense_step),
        "hbm_gbs_on_required_bytes": round(req_step / (ms_step * 1e-3) / 1e9, 1),
        "requested_bytes_per_step": int(requested_step if lay == "column" else req_step),
        "hbm_gbs_on_requested_bytes": round((requested_step if lay == "column" else req_step) / (ms_step * 1e-3) / 1e9, 1),
        "channel_major_stage1": {k: bool(v) for k, v in col.channel_major.items()},
        "dense_gemv_us_per_linear": {k: round(v, 3) for k, v in dense_us.items()},
        "dense_gemv_gbs": round(dense_step / n_lin / (best_dense * 1e-6) / 1e9, 1),
        "speedup_vs_dense_gemv": round(best_dense / us_linear, 3),
        "ideal_speedup_bytes_ratio": round(dense_step / req_step, 3),
        "roofline": {"bound": "hbm", "kernel": kern, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_from_profiles(kern, label),
                     "us_per_launch": round(us_launch, 3), "bytes_per_launch": int(bytes_launch),
                     # what the launches ask memory for: the required bytes minus the kept channels' columns of
                     # S_r V_r^T on the layers whose stage 1 reads the channel-major copy (traffic is compared with this)
                     "requested_bytes_per_launch": int((requested_step if lay == "column" else req_step) / n_calls),
                     "launches_per_step": n_calls},
    }
    log(f"{label}: R-Sparse {us_linear:.2f} us/linear ({lay}, {res[lay]['launch_mode']}; "
        f"{ {k: v['us_per_linear'] for k, v in res.items()} }), {out['hbm_gbs_on_required_bytes']:.0f} GB/s; "
        f"dense {dense_us}; speed-up {out['speedup_vs_dense_gemv']:.2f}x")

    cpu = None
    if want_cpu:
        threads = min(oracle.max_threads(), os.cpu_count() or 1, 16)
        t_cpu, n = 0.0, 0
        t_begin = time.time()
        while time.time() - t_begin < 10.0 and n < 6000:             # about 10 s of CPU work
            for name, *_ in wl["linears"]:
                L = col.base[name]
                t1 = time.time()
                oracle.rsparse_linear(L.W16, L.U16, L.SV16, col.blocks[0][name][3], dt, dt, col.tau[name][args.sparsity],
                                      nthreads=threads)
                t_cpu += time.time() - t1
                n += 1
        cpu = {"value": round(t_cpu / n * 1e6, 1), "unit": "us", "cores": threads, "kind": "oracle",
               "sample": f"{n} R-Sparse linear calls (the {n_lin} linears of {label} in turn, batch 1, same tokens and "
                         f"thresholds as the GPU run), fp64 C oracle with OpenMP over outputs"}
    return out, cpu, col, strip


def leg_weights_4bit(col, args, mods, timers, base_us=None):
    """configs[1]'s three linears with 4-bit weights (Sec. 4.4): R-Sparse at two ranks and the dense 4-bit GEMV."""
    torch, np, rs, synth, oracle = mods
    timed, best = timers
    stream = torch.cuda.current_stream()
    blocks, dt = len(col.blocks), col.wl["dtype"]
    g0, u0, d0 = (col.blocks[0][n] for n in ("gate", "up", "down"))

    def us(fn, per=3.0):
        return round(best(fn, blocks)[0] * 1000.0 / per, 3)

    # 4-bit weights (Sec. 4.4), the same three linears
    q4 = {}
    xs = {0: g0[1], 1: g0[1], 2: d0[1]}
    ys = {0: g0[2], 1: u0[2], 2: d0[2]}
    names = ["gate", "up", "down"]
    for q_rank in (512, 64):
        q_ring = []
        for li, name in enumerate(names):
            Lq = col.base[name]
            Qc, Sc, Zc = synth.quantize_q4(synth.decode16(Lq.W16, dt), dt, 128)
            d_in, d_out = Lq.d_in, Lq.d_out
            for blk in range(blocks):
                cfg = rs.make_config(d_in, d_out, q_rank, col.tau[name][args.sparsity], dt, max_batch=1,
                                     dense_rowmajor=1 if q_rank == 512 else 0)
                q_ring.append((li, blk, rs.rsparse_prepare_q4(cfg, Qc, Sc, Zc, 128, Lq.U16[:, :q_rank], Lq.SV16[:q_rank])))
        q_ring.sort(key=lambda e: (e[1], e[0]))

        def pass_q4(sptr):
            for li, _, layer in q_ring:
                rs.rsparse_linear(layer, xs[li].data_ptr(), 1, ys[li].data_ptr(), sptr)

        def pass_q4_dense(sptr):
            for li, _, layer in q_ring:
                rs.rsparse_dense_ref(layer, xs[li].data_ptr(), 1, ys[li].data_ptr(), sptr)

        pass_q4(stream.cuda_stream)
        torch.cuda.synchronize()
        rbq = sum(rs.rsparse_required_bytes(l, 1, len(rs.rsparse_last_active(l, -1))) for _, _, l in q_ring) / len(q_ring)
        uq = us(pass_q4)
        q4[f"rsparse_rank{q_rank}"] = {"us_per_linear": uq, "required_bytes_per_linear": int(rbq),
                                       "gbs_required": round(rbq / (uq * 1e-6) / 1e9, 1)}
        if q_rank == 512:
            dbq = sum(rs.rsparse_dense_bytes(l, 1) for _, _, l in q_ring) / len(q_ring)
            ud = us(pass_q4_dense)                     # row-dot over row-major codes (the copy is kept at this rank)
            q4["dense_4bit_rowdot"] = {"us_per_linear": ud, "bytes_per_linear": int(dbq), "gbs": round(dbq / (ud * 1e-6) / 1e9, 1)}
            for _, _, layer in q_ring:
                rs.rsparse_set_tuning(layer, dense_kernel=1)
            uc = us(pass_q4_dense)                     # the channel-major kernel with every channel kept
            q4["dense_4bit_channel_major"] = {"us_per_linear": uc, "bytes_per_linear": int(dbq), "gbs": round(dbq / (uc * 1e-6) / 1e9, 1)}
            for _, _, layer in q_ring:
                rs.rsparse_set_tuning(layer)
            q4["speedup_rank512_vs_best_dense_4bit"] = round(min(ud, uc) / uq, 3)
        for _, _, layer in q_ring:
            layer.destroy()
    q4["note"] = ("configs[1]'s three linears with 4-bit weights (GPTQ format, groups of 128), batch 1, two launches per "
                  "linear" + (f"; compare us_per_linear with the 16-bit column-major value {base_us}" if base_us else ""))
    return q4


def extras_config1(col, args, mods, timers):
    """Side measurements on configs[1]'s column-major ring: sparsity sweep, two-launch form and its kernels alone,
    separate calls, hot cache, one-call latency, the gated MLP entry points, 4-bit weights, streaming reference."""
    torch, np, rs, synth, oracle = mods
    timed, best = timers
    stream = torch.cuda.current_stream()
    blocks, dt = len(col.blocks), col.wl["dtype"]
    ex = {}

    def us(fn, per=3.0):
        return round(best(fn, blocks)[0] * 1000.0 / per, 3)

    base_us = us(col.pass_fn())
    col.set_all(dense_kernel=2)
    dense = us(col.pass_fn(dense=True))
    col.set_all()
    sweep = {}
    for s in (0.4, 0.7):
        col.set_tau(s)
        col.pass_fn()(stream.cuda_stream)
        torch.cuda.synchronize()
        rb = sum(rs.rsparse_required_bytes(l, 1, len(rs.rsparse_last_active(l, -1))) for l in col.layers()) / (3.0 * blocks)
        u = us(col.pass_fn())
        sweep[f"{int(s * 100)}%"] = {"us_per_linear": u, "gbs_required": round(rb / (u * 1e-6) / 1e9, 1),
                                     "speedup_vs_dense_rowdot": round(dense / u, 3)}
    col.set_tau(args.sparsity)
    ex["sparsity_sweep"] = sweep
    col.set_all(launches=2)
    ex["us_per_linear_two_launches"] = us(col.pass_fn())
    col.set_all()
    ex["us_per_linear_separate_calls"] = us(col.pass_fn(separate=True))
    g0, u0, d0 = (col.blocks[0][n] for n in ("gate", "up", "down"))

    def pass_hot(sptr):              # the same three layers every step: weights partly served by the Infinity Cache
        for _ in range(blocks):
            rs.rsparse_linear_group([g0[0], u0[0]], g0[1].data_ptr(), 1, [g0[2].data_ptr(), u0[2].data_ptr()], sptr)
            rs.rsparse_linear(d0[0], d0[1].data_ptr(), 1, d0[2].data_ptr(), sptr)

    ex["us_per_linear_hot_cache_same_layers"] = us(pass_hot)
    lat = []
    for i in range(60):              # one call at a time: host launch + kernel + synchronize, wall clock
        layer, xd, yd, _ = col.blocks[i % blocks]["down"]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        rs.rsparse_linear(layer, xd.data_ptr(), 1, yd.data_ptr(), stream.cuda_stream)
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - t1) * 1e6)
    lat.sort()
    ex["us_single_call_latency_incl_launch_and_sync"] = {"median": round(lat[len(lat) // 2], 1), "min": round(lat[0], 1),
                                                         "layer": "down 11008 -> 4096, one call, host wall clock"}
    # the gated MLP entry points (Sec. 3.1)
    d_ff = 11008
    pair = synth.GateUpPair(d_ff, config=1, linear=2)
    gus = []
    for i in range(blocks):
        g, u = pair.tokens(1, offset=1 + i)
        gus.append((torch.from_numpy(synth.encode16(g, dt).view(np.int16)).cuda(),
                    torch.from_numpy(synth.encode16(u, dt).view(np.int16)).cuda()))
    hbuf = torch.zeros((1, d_ff), dtype=torch.int16, device="cuda")

    def pass_gated(sptr):
        for b, (gd, ud) in zip(col.blocks, gus):
            rs.rsparse_linear_gated(b["down"][0], gd.data_ptr(), ud.data_ptr(), 1, b["down"][2].data_ptr(), sptr)

    def pass_down_only(sptr):
        for b in col.blocks:
            rs.rsparse_linear(b["down"][0], b["down"][1].data_ptr(), 1, b["down"][2].data_ptr(), sptr)

    def pass_gate_up_fused(sptr):
        for b in col.blocks:
            rs.rsparse_mlp_gate_up(b["gate"][0], b["up"][0], b["gate"][1].data_ptr(), 1, hbuf.data_ptr(), sptr)

    def pass_gate_up_only(sptr):
        for b in col.blocks:
            rs.rsparse_linear_group([b["gate"][0], b["up"][0]], b["gate"][1].data_ptr(), 1,
                                    [b["gate"][2].data_ptr(), b["up"][2].data_ptr()], sptr)

    ex["gate_up_with_activation_us"] = {"one_launch": us(pass_gate_up_fused, 1.0), "projections_only": us(pass_gate_up_only, 1.0),
                                        "note": "gate + up (2 x 4096 -> 11008): rsparse_mlp_gate_up (H = silu(g) * u stored by the "
                                                "kernel's finish) against the two projections alone"}
    ex["down_projection_gated_input_us"] = {"gated": us(pass_gated, 1.0), "plain_input": us(pass_down_only, 1.0),
                                            "note": "11008 -> 4096: rsparse_linear_gated (x = round(silu(g) * u) by one small "
                                                    "launch, then the layer) against rsparse_linear on a ready input"}
    ex["weights_4bit"] = leg_weights_4bit(col, args, mods, timers, base_us)
    # what this card streams at this launch size: library kernels over a ring of buffers of one launch's size
    n_el = int(sum(rs.rsparse_required_bytes(l, 1, len(rs.rsparse_last_active(l, -1))) for l in col.layers()) / (2 * blocks)) // 4
    srcs = [torch.ones(n_el, dtype=torch.float32, device="cuda") for _ in range(12)]
    dst = torch.empty(n_el, dtype=torch.float32, device="cuda")

    def time_ring(fn, reps=20):
        for t_ in srcs:
            fn(t_)
        torch.cuda.synchronize()
        b_ = 1e30
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                for t_ in srcs:
                    fn(t_)
            e1.record(stream)
            torch.cuda.synchronize()
            b_ = min(b_, e0.elapsed_time(e1) * 1e-3 / (reps * len(srcs)))
        return b_

    t_copy, t_read = time_ring(lambda t_: dst.copy_(t_)), time_ring(lambda t_: torch.sum(t_))
    ex["same_size_streaming_reference"] = {
        "bytes": n_el * 4, "copy_us": round(t_copy * 1e6, 2), "copy_gbs_read_plus_write": round(2 * n_el * 4 / t_copy / 1e9, 1),
        "read_sum_us": round(t_read * 1e6, 2), "read_sum_gbs": round(n_el * 4 / t_read / 1e9, 1),
        "note": "torch copy_ / sum over a ring of 12 buffers of one configs[1] launch's size; per-call time includes the launch"}
    return ex


def pmc_pass(label, cfg_no, args, mods):
    """For rocprofv3 --pmc / --kernel-trace: one 256 MiB device copy of known size (calibrates FETCH_SIZE / WRITE_SIZE),
    then 3 eager ring passes of R-Sparse on both layouts and of the dense row-dot baseline; no timing, no graphs."""
    torch, np, rs, synth, oracle = mods
    wl = workloads(synth)[label]
    stream = torch.cuda.current_stream()
    a = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")     # 256 MiB
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    b.copy_(a)
    torch.cuda.synchronize()
    col = Ring(wl, cfg_no, args.sparsity, 0, rs, synth, torch, np)
    strip = Ring(wl, cfg_no, args.sparsity, STRIP_COLS, rs, synth, torch, np, base=col.base)
    col.set_all(dense_kernel=2)
    for fn in (col.pass_fn(), strip.pass_fn(), col.pass_fn(dense=True)):
        for _ in range(3):
            fn(stream.cuda_stream)
            torch.cuda.synchronize()
    req = {}
    for ring, key in ((col, "column"), (strip, "strip")):
        req[key] = {name: rs.rsparse_required_bytes(e[0], 1, len(rs.rsparse_last_active(e[0], -1)))
                    for name, e in ring.blocks[0].items()}
    if args.pmc_mfma:
        dt = synth.BF16
        col.destroy()
        strip.destroy()
        # the matrix-core kernels at their largest shape: 8192 -> 28672, r = 1024, 32 tokens, eager launches
        Lb = synth.random_layer(8192, 28672, 1024, dt, seed=4242)
        srcb = synth.DModelInput(8192, config=4, linear=0)
        taub = rs.rsparse_calibrate_tau(synth.encode16(srcb.tokens(64, stream=synth.STREAM_CALIB), dt), dt, 0.5)
        big = [rs.rsparse_prepare_factors(rs.make_config(8192, 28672, 1024, taub, dt, max_batch=32, dense_rowmajor=1),
                                          Lb.W16, Lb.U16, Lb.SV16) for _ in range(2)]
        xb = torch.from_numpy(synth.encode16(srcb.tokens(32, offset=3), dt).view(np.int16)).cuda()
        yb = torch.zeros((32, 28672), dtype=torch.int16, device="cuda")
        for _ in range(2):
            for fn in (rs.rsparse_linear, rs.rsparse_dense_ref):
                for layer in big:
                    fn(layer, xb.data_ptr(), 32, yb.data_ptr(), stream.cuda_stream)
                    torch.cuda.synchronize()
        for layer in big:
            layer.destroy()
        # and the vector path at 4 tokens (4096 -> 11008, r = 512)
        L4 = synth.random_layer(4096, 11008, 512, dt, seed=4243)
        src4 = synth.DModelInput(4096, config=2, linear=0)
        tau4 = rs.rsparse_calibrate_tau(synth.encode16(src4.tokens(64, stream=synth.STREAM_CALIB), dt), dt, 0.5)
        four = [rs.rsparse_prepare_factors(rs.make_config(4096, 11008, 512, tau4, dt, max_batch=4, dense_rowmajor=1),
                                           L4.W16, L4.U16, L4.SV16) for _ in range(4)]
        x4 = torch.from_numpy(synth.encode16(src4.tokens(4, offset=3), dt).view(np.int16)).cuda()
        y4 = torch.zeros((4, 11008), dtype=torch.int16, device="cuda")
        for _ in range(3):
            for layer in four:
                rs.rsparse_linear(layer, x4.data_ptr(), 4, y4.data_ptr(), stream.cuda_stream)
                torch.cuda.synchronize()
        for layer in four:
            layer.destroy()
    print(json.dumps({"pmc_pass": label, "copy_bytes": int(a.numel() * 4), "required_bytes_block0": req,
                      "blocks": wl["blocks"], "calls": wl["calls"]}), flush=True)


def stamps_pass(label, cfg_no, args, mods):
    """Needs a library built with RSPARSE_STAMPS=1: per-wave phase time stamps of the strip kernel for every call of
    the workload (medians and spreads in microseconds after the launch's first wave starts); one JSON line."""
    torch, np, rs, synth, oracle = mods
    wl = workloads(synth)[label]
    stream = torch.cuda.current_stream()
    cap = 32768
    buf = torch.zeros(cap * 16, dtype=torch.int64, device="cuda")
    strip = Ring(wl, cfg_no, args.sparsity, STRIP_COLS, rs, synth, torch, np)
    run = strip.pass_fn()
    for _ in range(3):
        run(stream.cuda_stream)
    torch.cuda.synchronize()
    rs.rsparse_debug_stamps(buf.data_ptr(), cap)
    names_s = {1: "start", 11: "arguments", 12: "token_arrived", 2: "list_built", 13: "two_blocks_requested",
               3: "first_block_consumed", 4: "t_needed", 5: "t_there", 6: "rows_done", 7: "after_barrier", 8: "stored_or_added",
               9: "arrived_at_strip", 10: "finished_strip"}
    names_1 = {1: "start", 2: "token_staged", 3: "dots_done", 4: "published", 5: "closed"}
    out = {}
    b = strip.blocks[-1]
    for call in wl["calls"]:
        # the launch before this one keeps the pipeline as in the timed runs; the call's records are read after it alone
        run(stream.cuda_stream)
        torch.cuda.synchronize()
        buf.zero_()
        es = [b[n] for n in call]
        if len(call) == 1:
            rs.rsparse_linear(es[0][0], es[0][1].data_ptr(), 1, es[0][2].data_ptr(), stream.cuda_stream)
        else:
            rs.rsparse_linear_group([e[0] for e in es], es[0][1].data_ptr(), 1, [e[2].data_ptr() for e in es], stream.cuda_stream)
        torch.cuda.synchronize()
        a = buf.cpu().numpy().view(np.uint64).reshape(cap, 16)
        a = a[a[:, 1] != 0]
        kind = (a[:, 0] & 0xff).astype(int)
        t0 = float(a[:, 1].min())
        rec = {"waves": int(len(a)), "strip_waves": int((kind != 1).sum()), "stage1_waves": int((kind == 1).sum()),
               "rows_per_strip_wave_median": float(np.median(a[kind != 1, 15])) if (kind != 1).any() else 0.0}
        for tag, sel, names in (("strip", kind != 1, names_s), ("stage1", kind == 1, names_1)):
            for w_, nm in names.items():
                col_ = a[sel, w_].astype(np.float64)
                col_ = (col_[col_ != 0] - t0) / 100.0
                if len(col_):
                    rec[f"{tag}.{nm}"] = {"p10": round(float(np.percentile(col_, 10)), 2), "median": round(float(np.median(col_)), 2),
                                          "p90": round(float(np.percentile(col_, 90)), 2), "max": round(float(col_.max()), 2)}
        out["+".join(call)] = rec
    rs.rsparse_debug_stamps(0, 0)
    print(json.dumps({"stamps": label, "strip_cols": STRIP_COLS, "unit": "us after the launch's first wave started",
                      "calls": out}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sparsity", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements (configs[1] extras, the row-major stage-1 variant of configs[4])")
    ap.add_argument("--only", default="", help="comma-separated workloads to run (default: all three)")
    ap.add_argument("--eager", action="store_true", help="time eager launches only (no graph replay)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead: other shapes and batch sizes (R-Sparse vs dense per linear); one JSON line with key 'sweep'")
    ap.add_argument("--q4-pass", action="store_true", help="instead: only the 4-bit legs on configs[1]; one JSON line")
    ap.add_argument("--pmc-mfma", action="store_true",
                    help="with --pmc-pass: also the matrix-core kernels at 8192 -> 28672, 32 tokens, and the vector path at 4 tokens")
    ap.add_argument("--fast-layers", action="store_true", help="accepted and ignored (i.i.d. operands are what every mode uses)")
    ap.add_argument("--pmc-pass", default="", nargs="?", const="configs[1]", metavar="WORKLOAD",
                    help="for rocprofv3 --pmc / --kernel-trace: a 256 MiB copy of known size, then 3 eager passes of the "
                         "workload (e.g. 'configs[4]') with R-Sparse (both layouts) and the dense baseline; no timing")
    ap.add_argument("--stamps", default="", metavar="WORKLOAD",
                    help="per-wave phase time stamps of the strip kernel on the workload (needs a RSPARSE_STAMPS=1 build)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (one MI355X); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.stamps:                 # the measurement build, beside the ordinary one
        os.environ["RSPARSE_LIB"] = os.path.join(ROOT, "paper_2504_19449_amd", "librsparse_stamps.so")
        if not os.path.exists(os.environ["RSPARSE_LIB"]):
            print("bench.py --stamps: build it first with `python -m paper_2504_19449_amd.build --stamps`", file=sys.stderr)
            sys.exit(2)

    import numpy as np
    import torch

    import paper_2504_19449_amd as rs
    from paper_2504_19449_amd import build as lib_build
    from paper_2504_19449_amd import synth

    if not os.path.exists(rs.library_path()):
        lib_build.build(force=True)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    import oracle
    mods = (torch, np, rs, synth, oracle)
    cfg_no = {"configs[0]": 0, "configs[1]": 1, "configs[4]": 4}

    if args.sweep:
        print(json.dumps({"decoder_layer": decoder_layer_sweep(torch, np, rs, synth),
                          "sweep": shape_batch_sweep(args, torch, np, rs, synth)}), flush=True)
        return
    if args.pmc_pass:
        pmc_pass(args.pmc_pass, cfg_no[args.pmc_pass], args, mods)
        return
    if args.q4_pass:
        col = Ring(workloads(synth)["configs[1]"], 1, args.sparsity, 0, rs, synth, torch, np)
        print(json.dumps({"weights_4bit": leg_weights_4bit(col, args, mods, make_timer(torch, args))}), flush=True)
        return
    if args.stamps:
        stamps_pass(args.stamps, cfg_no[args.stamps], args, mods)
        return

    timers = make_timer(torch, args)
    only = [w for w in args.only.split(",") if w] or ["configs[4]", "configs[1]", "configs[0]"]
    results, cpu, extras = {}, None, {}
    for label in ("configs[4]", "configs[1]", "configs[0]"):
        if label not in only:
            continue
        want_cpu = not args.no_cpu_baseline and label == only[0]
        out, c, col, strip = measure_workload(label, cfg_no[label], args, mods, timers, want_cpu)
        results[label] = out
        cpu = c if c is not None else cpu
        strip.destroy()
        if label == "configs[1]" and not args.no_extras:
            extras = extras_config1(col, args, mods, timers)
            log(f"configs[1] extras: { {k: v for k, v in extras.items() if k != 'weights_4bit'} }")
        col.destroy()

    head = results[only[0]]
    line = {
        "metric": "us_per_rsparse_linear_batch1", "value": head["us_per_linear"], "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if only[0] != "configs[0]" else "f16", "data": "synthetic (i.i.d. weights and factors of the workload's scales; "
        "heavy-tailed Laplace x LogNormal tokens with 8 outlier channels, SiLU(g)*u for down projections)",
        "config": {"workload": head["workload"] + f"; ring of distinct layers >= 1 GiB; {head['layout']} layout, "
                               f"{'plain stream launches' if head['launch_mode'] == 'eager' else 'HIP-graph replay'}; "
                               f"median of {REPEATS} brackets of `steps` steps",
                   "batch": 1, "sparsity": args.sparsity, "layout": head["layout"], "launch_mode": head["launch_mode"]},
        "hbm_gbs_on_required_bytes": head["hbm_gbs_on_required_bytes"],
        "hbm_frac_on_required_bytes": round(head["hbm_gbs_on_required_bytes"] / HBM_PEAK_GBS, 4),
        "dense_gemv_us": head["dense_gemv_us_per_linear"], "speedup_vs_dense_gemv": head["speedup_vs_dense_gemv"],
        "roofline": head["roofline"], "cpu_baseline": cpu,
        "workloads": results,
    }
    if extras:
        line["configs[1]_extras"] = extras
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
