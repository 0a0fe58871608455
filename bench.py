#!/usr/bin/env python3
"""Throughput of the LoRDBA adapter forward branch on one MI355X.

A step is one lordba_forward call (the whole hot path: bit-unpack, s_in scaling + sign(A) reduction,
s_rank scaling, sign(B) expansion, s_out epilogue added to y_base) on one batch of seeded synthetic
inputs that are already resident in HBM.  The default workload is the LLaMA-2-7B attention-projection
shape d_in = d_out = 4096, r = 16, T = 2048.  Steps cycle through enough distinct (x, y_base, y_out)
buffer sets that the 256 MB Infinity Cache cannot hold them, so the reported GB/s is HBM traffic.

Prints one JSON line: metric/value (tokens/s), ms_per_step, a `roofline` object for the kernel
(algorithmic bytes per launch / average launch duration from HIP events on the launch stream, against
the 8 TB/s HBM peak), and a `cpu_baseline` object (the fp64 CPU oracle timed on the host cores).

Two further workloads report what the single-shape line cannot:
  --workload c5_model   one step = the 280 adapter calls of a 40-layer LLaMA-2-13B pass at T = 8192
                        (280 distinct adapters resident, three rotating activation sets); value = model-level tokens/s
  --workload c4_sweep   the decode-size shapes r in {8,16,32,64} x T in {1,8,64}: microseconds per call beside the
                        launch-to-launch floor of an empty kernel on the same stream
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
# bench.py cannot read hardware counters itself: `traffic` (HBM bytes per call from rocprofv3 FETCH_SIZE + WRITE_SIZE) is
# looked up in profiles/hbm_traffic.json, which paper_2605_24058_amd/traffic_profile.py writes from the counter files and
# stamps with a hash of the kernel sources; it is null, with the reason, once those sources have changed.
CACHE_BYTES = 256 << 20        # Infinity Cache
REPS = 7                       # repetitions of the timed region; the median one is reported

WORKLOADS = {}


def _shape(name):
    """A workload by name, or any shape written T,d_in,d_out,r (for sweeps and counter runs)."""
    from paper_2605_24058_amd import inputs
    parts = name.split(",")
    if len(parts) == 4 and all(p.isdigit() for p in parts):
        T, d_in, d_out, r = (int(p) for p in parts)
        return inputs.Shape("shape_%dx%d_r%d_T%d" % (d_in, d_out, r, T), T, d_in, d_out, r)
    return _workloads()[name]


def _workloads():
    from paper_2605_24058_amd import inputs
    if not WORKLOADS:
        for sh in [inputs.C1, inputs.C2, inputs.C3_UP, inputs.C3_DOWN, inputs.C5_Q, inputs.C5_UP, inputs.C5_DOWN] + inputs.C4:
            WORKLOADS[sh.name] = sh
        WORKLOADS.update({"c1": inputs.C1, "c2": inputs.C2, "c3_up": inputs.C3_UP, "c3_down": inputs.C3_DOWN,
                          "c5_q": inputs.C5_Q, "c5_up": inputs.C5_UP, "c5_down": inputs.C5_DOWN})
    return WORKLOADS


WARM_SECONDS = 0.06            # untimed replays of the timed region before the first timed one: the clocks ramp up


def timed(fn, K, W, graph, reps=1, warm_s=WARM_SECONDS):
    """Runs fn(0..K-1) as the timed region `reps` times.  Returns (microseconds per step of each repetition from HIP
    events on the launch stream, wall-clock seconds of each repetition).  Before the first timed repetition the region is
    run untimed for at least `warm_s` seconds, whatever W and K are: on a box that has been idle the first ~50 ms of work
    run at lower clocks, and a region of a few dozen 10-microsecond launches would otherwise be measured inside that ramp."""
    import torch
    for i in range(W):
        fn(i)
    torch.cuda.synchronize()
    us, walls = [], []
    if graph:
        # The K launches of the timed region are captured once and replayed: same kernels, same buffers, no host
        # launch cost between them.  Only kernel launches are captured (no memset nodes).
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(K):
                fn(i)
        g.replay()               # untimed replay: graph upload
        run = g.replay
    else:
        def run():
            for i in range(K):
                fn(i)
    torch.cuda.synchronize()
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < warm_s:
        run()
        torch.cuda.synchronize()
    for _ in range(reps):
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a0.record()
        run()
        a1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        us.append(a0.elapsed_time(a1) * 1e3 / K)
        walls.append(t1 - t0)
    return us, walls


def _median_index(v):
    """Index of the median repetition (the lower of the two middle ones for an even count): a figure that was measured."""
    order = sorted(range(len(v)), key=lambda i: v[i])
    return order[(len(v) - 1) // 2]


def _median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


def bench_c4_sweep(args):
    """Decode-size calls: a roofline fraction says nothing at <= 1.7 MB per call, so the line reports microseconds per
    call beside the launch-to-launch floor of the stream (an empty kernel in the same graph-replay harness)."""
    import numpy as np
    import torch
    from paper_2605_24058_amd import binding, inputs
    ref = binding.load_bench_library()
    cur = lambda: torch.cuda.current_stream().cuda_stream
    K, W = args.steps, args.warmup
    use_graph = not args.no_graph

    def empty_step(i):
        assert ref.lordba_bench_empty(cur()) == 0

    torch.manual_seed(args.seed)
    floor_us, _ = timed(empty_step, K, W, use_graph, reps=5)
    rows, total_wall, total_tok = [], 0.0, 0
    for sh in inputs.C4:
        sets = 16                                   # distinct activation sets: inputs come from HBM / far cache, not L2
        host = inputs.make_inputs_for(sh, args.seed)
        dev = binding.to_device(host)
        xs = [dev["x"]] + [torch.randn_like(dev["x"]) for _ in range(sets - 1)]
        ybs = [dev["y_base"]] + [torch.randn_like(dev["y_base"]) for _ in range(sets - 1)]
        youts = [torch.empty_like(y) for y in ybs]

        def step(i):
            s = i % sets
            binding.lordba_forward(xs[s], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                   ybs[s], y_out=youts[s], algo=args.algo, check=False)

        us, walls = timed(step, K, W, use_graph, reps=5)
        total_wall += walls[_median_index(us)]
        total_tok += sh.T * K
        rows.append({"r": sh.r, "T": sh.T, "us_per_call": _median(us), "tokens_per_s": sh.T / (_median(us) * 1e-6),
                     "algorithmic_bytes": sh.algorithmic_bytes()})
    out = {"metric": "adapter-branch microseconds per call at d=4096, r in {8,16,32,64}, T in {1,8,64}",
           "value": total_tok / total_wall, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": total_wall * 1e3 / (K * len(rows)), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "io_dtype": "f16", "data": "synthetic",
           "config": {"workload": "c4_sweep", "d_in": 4096, "d_out": 4096, "launch": "hip_graph" if use_graph else "eager",
                      "algo": args.algo, "seed": args.seed, "repetitions": 5, "statistic": "median"},
           "launch_floor_us": _median(floor_us), "calls": rows}
    print(json.dumps(out))


def bench_c5_model(args):
    """All 280 adapter calls of one LLaMA-2-13B pass (40 layers x q, k, v, o, gate, up, down) at T = 8192."""
    import numpy as np
    import torch
    from paper_2605_24058_amd import binding, inputs
    K, W = args.steps, args.warmup
    use_graph = not args.no_graph
    T = inputs.C5_Q.T
    nsets = 3
    # ---- 280 adapters, all resident ------------------------------------------------------------------------------
    adapters = []
    for layer, name, sh, seed in inputs.c5_adapter_seeds(args.seed):
        h = inputs.make_adapter(seed, sh.d_in, sh.d_out, sh.r)
        pA, pB = binding.lordba_pack_signs(h["signsA"], h["signsB"])
        d = {k: torch.from_numpy(h[k]).cuda() for k in ("s_in", "s_rank", "s_out")}
        d["packedA"] = torch.from_numpy(pA.view(np.int32)).cuda()
        d["packedB"] = torch.from_numpy(pB.view(np.int32)).cuda()
        adapters.append((layer, name, sh, h, d))
    # ---- three rotating activation sets, each with buffers of both widths -----------------------------------------
    widths = sorted({sh.d_in for *_, sh, _, _ in adapters} | {sh.d_out for *_, sh, _, _ in adapters})
    host_sets, dev_sets = [], []
    for s in range(nsets):
        hs, ds = {}, {}
        for w in widths:
            act = inputs.make_activations(args.seed + 7919 * (s + 1) + w, T, w, w)
            hs[w] = act
            ds[w] = {"x": torch.from_numpy(act["x"]).cuda(), "y_base": torch.from_numpy(act["y_base"]).cuda()}
            ds[w]["y_out"] = torch.empty_like(ds[w]["y_base"])
        host_sets.append(hs)
        dev_sets.append(ds)
    torch.cuda.synchronize()
    ncalls = len(adapters)

    def call(c):
        layer, name, sh, h, d = adapters[c]
        s = c % nsets
        return binding.lordba_forward(dev_sets[s][sh.d_in]["x"], d["packedA"], d["packedB"], d["s_in"], d["s_rank"], d["s_out"],
                                      dev_sets[s][sh.d_out]["y_base"], y_out=dev_sets[s][sh.d_out]["y_out"],
                                      algo=args.algo, check=False)

    def model_pass(i):
        for c in range(ncalls):
            call(c)

    us, walls = timed(model_pass, K, W, use_graph, reps=3)
    pass_us, wall = us[_median_index(us)], walls[_median_index(us)]
    alg_bytes = sum(sh.algorithmic_bytes() for *_, sh, _, _ in adapters)
    achieved = alg_bytes / (pass_us * 1e-6) / 1e9
    out = {"metric": "model-level adapter-branch tokens/s over the 280 adapter calls of LLaMA-2-13B at T=8192",
           "value": T * K / wall, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": wall * 1e3 / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "io_dtype": "f16", "data": "synthetic",
           "config": {"workload": "c5_model", "T": T, "r": 16, "layers": inputs.C5_LAYERS, "calls_per_step": ncalls,
                      "activation_sets": nsets, "launch": "hip_graph" if use_graph else "eager", "algo": args.algo,
                      "seed": args.seed},
           "achieved_hbm_gbs": achieved, "hbm_peak_gbs": HBM_PEAK_GBS,
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel_us": pass_us / ncalls,
                        "kernel_us_repetitions": [u / ncalls for u in us],
                        "algorithmic_bytes": alg_bytes, "note": "all 280 launches of a pass taken together; median of 3 repetitions"}}
    if not args.no_cpu_baseline:
        # The oracle on every 64th token row of all 280 projections; the same rows are the parity check.
        import oracle
        cores = oracle.available_cores()
        idx = np.arange(0, T, 64)
        didx = torch.from_numpy(idx).cuda()
        worst, cpu_s = 0.0, 0.0
        for c in range(ncalls):
            layer, name, sh, h, d = adapters[c]
            s = c % nsets
            xh, ybh = host_sets[s][sh.d_in]["x"][idx], host_sets[s][sh.d_out]["y_base"][idx]
            c0 = time.perf_counter()
            want = oracle.forward(xh, h["signsA"], h["signsB"], h["s_in"], h["s_rank"], h["s_out"], ybh, nthreads=cores)
            cpu_s += time.perf_counter() - c0
            got = call(c)[didx]
            worst = max(worst, float(oracle.row_rel_l2(got.cpu().numpy().astype(np.float64), want).max()))
        out["cpu_baseline"] = {"value": len(idx) / cpu_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": "every 64th token row (%d of %d) through all %d projections" % (len(idx), T, ncalls)}
        out["parity_max_row_rel_l2"] = worst
        out["parity_ok"] = bool(worst <= 1e-3)
    print(json.dumps(out))


def backward_algorithmic_bytes(sh):
    """What one backward call of the branch must move: x, g, dx_base read and dx written once (fp16); the three packed
    carriers it takes; the fp16 scales; the fp32 latents read and the fp32 gradients of latents and scales written."""
    act = 2 * sh.T * (3 * sh.d_in + sh.d_out)
    carriers = (sh.r * (2 * sh.d_in + sh.d_out) + 7) // 8
    scales = 2 * (sh.d_in + sh.r + sh.d_out)
    latents = 4 * sh.r * (sh.d_in + sh.d_out)
    grads = latents + 4 * (sh.d_in + sh.r + sh.d_out)
    return act + carriers + scales + latents + grads


def bench_backward(args):
    """One step = one lordba_backward call (input gradient, scale gradients, latent-carrier gradients through the
    smooth-sign factor) on HBM-resident inputs, cycling through enough buffer sets to defeat the Infinity Cache."""
    import numpy as np
    import torch
    from paper_2605_24058_amd import binding, inputs, traffic_profile
    K, W = args.steps, args.warmup
    use_graph = not args.no_graph
    sh = _shape(args.workload)
    per_set = 2 * sh.T * (3 * sh.d_in + sh.d_out)
    sets = args.sets if args.sets > 0 else max(2, -(-2 * CACHE_BYTES // per_set) + 1)
    host0 = inputs.make_backward_inputs(args.seed, sh.T, sh.d_in, sh.d_out, sh.r)
    pA, _ = binding.lordba_pack_signs(host0["signsA"], host0["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(host0["signsA"], host0["signsB"])
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dev = {k: cu(host0[k]) for k in ("s_in", "s_rank", "s_out", "latA", "latB")}
    dev.update(pA=cu(pA.view(np.int32)), pAt=cu(pAt.view(np.int32)), pBt=cu(pBt.view(np.int32)))
    xs, gs, dxbs, dxs = [], [], [], []
    for s_ in range(sets):
        h = host0 if s_ == 0 else inputs.make_backward_inputs(args.seed + 1000 * s_, sh.T, sh.d_in, sh.d_out, sh.r)
        xs.append(cu(h["x"])); gs.append(cu(h["g"])); dxbs.append(cu(h["dx_base"])); dxs.append(torch.empty_like(dxbs[-1]))
    ws = torch.empty(binding.lordba_backward_multi_workspace_bytes(sh.T, sh.d_in, sh.d_out, sh.r, args.ell), dtype=torch.uint8, device="cuda")
    kept = [None] * sets
    if args.keep_t:   # the rank-r intermediate of each set, kept by the training forward (outside the timed region)
        _, pB = binding.lordba_pack_signs(host0["signsA"], host0["signsB"])
        dev["pB"] = cu(pB.view(np.int32))
        for s_ in range(sets):
            _, kept[s_] = binding.lordba_forward_save_t(xs[s_], dev["pA"], dev["pB"], dev["s_in"], dev["s_rank"], dev["s_out"])
    torch.cuda.synchronize()
    outs = {}

    y_bases = [cu(host0["y_base"]) if s_ == 0 else torch.randn_like(gs[0]) for s_ in range(sets)] if args.train_step else None
    y_outs = [torch.empty_like(y) for y in y_bases] if args.train_step else None
    t_bufs = [torch.empty((sh.r, binding.saved_t_stride(sh.T)), dtype=torch.float32, device="cuda") for _ in range(sets)] if args.train_step else None

    def train_step(i):
        """One training step of the branch: sign and pack the latents, forward (keeping t), backward."""
        s_ = i % sets
        pA_, pB_, pAt_, pBt_ = binding.lordba_pack_latents(dev["latA"], dev["latB"])
        binding.lordba_forward_save_t(xs[s_], pA_, pB_, dev["s_in"], dev["s_rank"], dev["s_out"], y_bases[s_], y_out=y_outs[s_],
                                      t_out=t_bufs[s_])
        outs[s_] = binding.lordba_backward(xs[s_], gs[s_], pA_, pAt_, pBt_, dev["s_in"], dev["s_rank"], dev["s_out"], dev["latA"],
                                           dev["latB"], args.kappa, dx_base=dxbs[s_], dx=dxs[s_], workspace=ws, check=False,
                                           t_saved=t_bufs[s_])

    ell = args.ell
    if ell > 1:   # several envelopes over the same carriers: lordba_backward_multi (t is always recomputed there)
        assert not args.train_step and not args.keep_t, "--ell > 1 goes with the plain --backward mode"
        env = inputs.make_envelopes(args.seed, sh.d_in, sh.d_out, sh.r, ell)
        dev.update({k: cu(env[k]) for k in ("s_in", "s_rank", "s_out")})

    def step(i):
        if args.train_step:
            return train_step(i)
        s_ = i % sets
        if ell > 1:
            outs[s_] = binding.lordba_backward_multi(xs[s_], gs[s_], dev["pA"], dev["pAt"], dev["pBt"], dev["s_in"], dev["s_rank"],
                                                     dev["s_out"], dev["latA"], dev["latB"], args.kappa, dx_base=dxbs[s_], dx=dxs[s_],
                                                     workspace=ws)
            return
        outs[s_] = binding.lordba_backward(xs[s_], gs[s_], dev["pA"], dev["pAt"], dev["pBt"], dev["s_in"], dev["s_rank"],
                                           dev["s_out"], dev["latA"], dev["latB"], args.kappa, dx_base=dxbs[s_], dx=dxs[s_],
                                           workspace=ws, check=False, t_saved=kept[s_])

    reps_us, walls = timed(step, K, max(W, sets), use_graph, reps=5)
    call_us, wall_s = reps_us[_median_index(reps_us)], walls[_median_index(reps_us)]   # the median repetition
    alg = backward_algorithmic_bytes(sh)
    alg += (ell - 1) * (2 + 4) * (sh.d_in + sh.r + sh.d_out)     # further envelopes: fp16 scales read, fp32 scale gradients written
    if args.train_step:   # + the forward call + reading the latents and writing the four packed carriers
        alg += sh.algorithmic_bytes() + 4 * sh.T * sh.r + 4 * sh.r * (sh.d_in + sh.d_out) + 4 * ((sh.r * (sh.d_in + sh.d_out) + 7) // 8)
    achieved = alg / (call_us * 1e-6) / 1e9
    traffic, traffic_note = (None, "not measured for this mode") if (args.train_step or ell > 1) else \
        traffic_profile.lookup("lordba_backward", sh.name, "t kept" if args.keep_t else "t recomputed")
    out = {"metric": ("adapter-branch training step (pack latents, forward, backward) tokens/s and achieved HBM GB/s" if args.train_step else
                      "adapter-branch backward (dx, scale and latent-carrier gradients) tokens/s and achieved HBM GB/s"),
           "value": sh.T * K / wall_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": wall_s * 1e3 / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "io_dtype": "f16", "data": "synthetic",
           "config": {"workload": sh.name, "pass": "train_step" if args.train_step else "backward", "T": sh.T, "d_in": sh.d_in, "d_out": sh.d_out, "r": sh.r,
                      "ell": ell, "kappa": args.kappa, "t": "kept by the forward pass" if args.keep_t else "recomputed from x", "buffer_sets": sets, "launch": "hip_graph" if use_graph else "eager", "seed": args.seed},
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                        "traffic": traffic, "traffic_source": traffic_note,
                        "kernel_us": call_us, "kernel_us_repetitions": reps_us, "algorithmic_bytes": alg,
                        "note": "all kernels of one call taken together (dx + du, t unless kept, wgrad, finish)"}}
    if not args.no_cpu_baseline:
        import oracle
        rows = min(sh.T, 256)
        c0 = time.perf_counter()
        if ell > 1:
            want = oracle.backward_multi(host0["x"][:rows], host0["g"][:rows], host0["signsA"], host0["signsB"], env["s_in"],
                                         env["s_rank"], env["s_out"], host0["latA"], host0["latB"], args.kappa, host0["dx_base"][:rows])
        else:
            want = oracle.backward(host0["x"][:rows], host0["g"][:rows], host0["signsA"], host0["signsB"], host0["s_in"],
                                   host0["s_rank"], host0["s_out"], host0["latA"], host0["latB"], args.kappa, host0["dx_base"][:rows])
        c1 = time.perf_counter()
        step(0)
        torch.cuda.synchronize()
        if args.train_step:   # the forward output of the step, same rows
            ywant = oracle.forward(host0["x"][:rows], host0["signsA"], host0["signsB"], host0["s_in"], host0["s_rank"], host0["s_out"],
                                   host0["y_base"][:rows])
            out["parity_max_row_rel_l2_y"] = float(oracle.row_rel_l2(y_outs[0][:rows].cpu().numpy().astype(np.float64), ywant).max())
        err = float(oracle.row_rel_l2(dxs[0][:rows].cpu().numpy().astype(np.float64), want["dx"]).max())
        out["cpu_baseline"] = {"value": rows / (c1 - c0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": "the first %d of %d token rows of the same workload, one host thread" % (rows, sh.T)}
        out["parity_max_row_rel_l2_dx"] = err
        out["parity_ok"] = bool(err <= 1e-3)
    print(json.dumps(out))


FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X published fp64 vector peak


def ptq_algorithmic_flops(N, M, R, r0, sweeps):
    """fp64 operations of `sweeps` sweeps of the consensus ADMM with the target kept factored (a multiply-add counts as
    two).  Per row of either side and sweep: the Tikhonov step (right-hand side 2 R r0, matrix R^2, Cholesky R^3/3,
    two triangular solves 2 R^2), the closed-form scale (2 R r0 + 2 R^2), and the row's share of the two Gram pairs its
    side contributes per sweep (2 x 2 (R^2 + R r0)); plus the R x R beta solve and the sign / dual update (6 per entry)."""
    per_row = (2 * R * r0 + R * R + R ** 3 / 3.0 + 2 * R * R) + (2 * R * r0 + 2 * R * R) + 4 * (R * R + R * r0) + 6 * R
    return sweeps * ((N + M) * per_row + R ** 3 / 3.0 + 4 * R * R)


def bench_ptq(args):
    """One step = one lordba_ptq call: the update of one 4096 x 4096 projection (rank-16 fp16 factors, resident in HBM)
    quantised into a LoRDBA adapter of carrier rank 16 with the paper's settings (K = 100, (tau, mu) = (2, 10))."""
    import numpy as np
    import torch
    from paper_2605_24058_amd import binding, inputs
    N, M, R, r0 = (int(v) for v in args.ptq_shape.split(","))
    Kadmm = 100
    K, W = args.steps, args.warmup
    sets = 4
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    host = [inputs.make_ptq_inputs(args.seed + 1000 * s_, N, M, r0) for s_ in range(sets)]
    dev = [(cu(h["A_star"]), cu(h["B_star"])) for h in host]
    ws = torch.empty(binding.lordba_ptq_workspace_bytes(N, M, R, r0) // 8, dtype=torch.float64, device="cuda")
    outs = {}

    def step(i):
        s_ = i % sets
        outs[s_] = binding.lordba_ptq(dev[s_][0], dev[s_][1], R, K=Kadmm, workspace=ws)

    use_graph = not args.no_graph
    S = max(1, args.ptq_streams)
    C = args.ptq_chunk
    if S > 1 or C > 0:
        # Several projections at once: one call is a chain of short dependent launches that leaves most of the chip idle,
        # and it never waits for the device, so independent calls on separate streams (each with its own workspace and
        # outputs, each captured into its own HIP graph) overlap.  K calls are dealt round-robin to the S streams.
        # With --ptq-chunk C a run is enqueued in two pieces (lordba_ptq_sweeps): sweeps [0, C), then the host waits for
        # that stream, reads the end flag, and enqueues [C, K) only if the loop has not ended yet.
        streams = [torch.cuda.Stream() for _ in range(S)]
        graphs, rest, held = [], [], []
        first = (0, C) if C > 0 else (0, Kadmm)
        for j in range(S):
            A_, B_ = dev[j % sets]
            with torch.cuda.stream(streams[j]):
                o = binding.lordba_ptq(A_, B_, R, K=Kadmm, stream=streams[j])       # allocates outputs and workspace; warms up
                streams[j].synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=streams[j]):
                    binding.lordba_ptq(A_, B_, R, K=Kadmm, stream=streams[j], sweeps=first, out=o)
                g2 = None
                if C > 0:
                    g2 = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g2, stream=streams[j]):
                        binding.lordba_ptq(A_, B_, R, K=Kadmm, stream=streams[j], sweeps=(C, Kadmm), out=o)
            graphs.append(g); rest.append(g2); held.append(o)
            outs[j % sets] = o
        torch.cuda.synchronize()
        continued = 0

        def finish(j):
            nonlocal continued
            if C > 0:
                streams[j].synchronize()
                if held[j]["info"][1].item() == 0.0:      # the loop has not ended within the first piece
                    continued += 1
                    with torch.cuda.stream(streams[j]):
                        rest[j].replay()

        reps_us, walls = [], []
        for _ in range(3):
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            a0.record()
            for j in range(S):
                streams[j].wait_event(a0)
            for i in range(K):
                j = i % S
                if i >= S:
                    finish(j)                               # the call this stream was given a round ago
                with torch.cuda.stream(streams[j]):
                    graphs[j].replay()
            for j in range(min(S, K)):
                finish(j)
            for j in range(S):
                torch.cuda.current_stream().wait_stream(streams[j])
            a1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            reps_us.append(a0.elapsed_time(a1) * 1e3 / K)
            walls.append(t1 - t0)
    else:
        reps_us, walls = timed(step, K, W, use_graph, reps=3)
    torch.cuda.synchronize()
    call_us, wall_s = reps_us[_median_index(reps_us)], walls[_median_index(reps_us)]
    sweeps = [int(outs[s_]["info"][0].item()) for s_ in outs if not isinstance(s_, tuple)]
    mean_sweeps = sum(sweeps) / len(sweeps)
    flops = ptq_algorithmic_flops(N, M, R, r0, mean_sweeps)
    achieved = flops / (call_us * 1e-6) / 1e12
    out = {"metric": "PTQ-LoRDBA projections/s (one %d x %d update, rank-%d factors -> carrier rank %d, K = 100)" % (N, M, r0, R),
           "value": K / wall_s, "unit": "projections/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": wall_s * 1e3 / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f64", "io_dtype": "f16", "data": "synthetic",
           "config": {"workload": "ptq_%dx%d_R%d_r%d_K100" % (N, M, R, r0), "N": N, "M": M, "R": R, "r0": r0, "K": Kadmm, "tau": 2.0, "mu": 10.0,
                      "sweeps_run": sweeps, "launch": "hip_graph" if (use_graph or S > 1) else "eager", "concurrent_streams": S,
                      "pieces": ("[0, %d) then, after a look at the end flag, [%d, %d)" % (C, C, Kadmm)) if C > 0 else "one call", "seed": args.seed},
           "roofline": {"bound": "alu", "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "traffic": None, "kernel_us": call_us,
                        "kernel_us_repetitions": reps_us, "algorithmic_flops": flops,
                        "note": "all kernels of one call taken together; the call is a chain of dependent launches on "
                                "R x R and N x R operands and is bound by their latency, not by arithmetic or HBM"}}
    if not args.no_cpu_baseline:
        from oracle import ptq as P
        n = min(4096, N, M)           # the default projection whole: the dense oracle takes about 10 s on the GPU machine's host
        h = inputs.make_ptq_inputs(args.seed, n, n, r0)
        c0 = time.perf_counter()
        ref = P.ptq(h["A_star"], h["B_star"], R, K=Kadmm)
        c1 = time.perf_counter()
        got = binding.lordba_ptq(cu(h["A_star"]), cu(h["B_star"]), R, K=Kadmm)
        torch.cuda.synchronize()
        sA, sB = binding.lordba_unpack_signs(got["packedA"].cpu().numpy().view(np.uint32), got["packedB"].cpu().numpy().view(np.uint32), n, n, R)
        g1, g2, _ = P.canonical_gauge(sA.T.astype(np.float64), sB.T.astype(np.float64))
        r1, r2, _ = P.canonical_gauge(ref["B1"], ref["B2"])
        same = bool(np.array_equal(g1, r1) and np.array_equal(g2, r2) and int(got["info"][0].item()) == ref["sweeps"])
        err = max(float(np.linalg.norm(got[k].cpu().numpy() - ref[k]) / np.linalg.norm(ref[k])) for k in ("alpha", "beta", "gamma"))
        out["cpu_baseline"] = {"value": 1.0 / (c1 - c0), "unit": "projections/s of a %d x %d update" % (n, n), "cores": min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)), "kind": "oracle",
                               "sample": "one %d x %d update (the default workload's projection whole), same ranks and K; " % (n, n) +
                                         "numpy's threaded BLAS on all host cores"}
        out["parity_signs_and_sweeps_exact"] = same
        out["parity_max_rel_l2_scales"] = err
        out["parity_ok"] = bool(same and err <= 1e-8)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c2",
                    help="c1, c2 (default), c3_up, c3_down, c5_q, c5_up, c5_down, a full shape name, or T,d_in,d_out,r; c5_model (the 280 adapter "
                         "calls of a LLaMA-2-13B pass); c4_sweep (decode sizes, microseconds per call)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--ell", type=int, default=1, help="scale envelopes over the same carriers (1 = lordba_forward; "
                    "2..4 = lordba_forward_multi); single-shape workloads only")
    ap.add_argument("--adapters", type=int, default=0, help="serve the batch with a pool of this many adapters through "
                    "lordba_forward_batched (0 = one adapter, lordba_forward; with --ell 2..4: lordba_forward_batched_multi); single-shape workloads")
    ap.add_argument("--id-pattern", choices=["segments", "decode", "mixed"], default="segments",
                    help="adapter index per token row: sorted segments (prefill of several requests), independent draws "
                         "(decode, one token per request) or segments with rows that have no adapter")
    ap.add_argument("--backward", action="store_true", help="time lordba_backward (the branch's backward pass in training) "
                    "instead of the forward call; single-shape workloads only")
    ap.add_argument("--train-step", action="store_true", help="time one training step of the branch: lordba_pack_latents, "
                    "lordba_forward_save_t, lordba_backward with the kept t (implies --backward)")
    ap.add_argument("--ptq", action="store_true", help="time lordba_ptq (post-training quantisation of one 4096 x 4096 update) "
                    "instead of the forward pass")
    ap.add_argument("--ptq-streams", type=int, default=1, help="--ptq: this many projections in flight at once, one stream and "
                    "one HIP graph each")
    ap.add_argument("--ptq-chunk", type=int, default=32, help="--ptq: enqueue the first this many sweeps, wait, and enqueue the rest "
                    "only if the loop has not ended (lordba_ptq_sweeps); 0 = one call of all K sweeps that never waits")
    ap.add_argument("--ptq-shape", default="4096,4096,16,16", help="--ptq: N,M,R,r0 (update N x M, carrier rank R, factor rank r0)")
    ap.add_argument("--keep-t", action="store_true", help="--backward: pass the rank-r intermediate kept by "
                    "lordba_forward_save_t instead of letting lordba_backward recompute it from x")
    ap.add_argument("--kappa", type=float, default=100.0, help="temperature of the smooth-sign factor (--backward)")
    ap.add_argument("--sets", type=int, default=0, help="distinct buffer sets to cycle through (0 = enough to defeat the cache)")
    ap.add_argument("--algo", type=int, default=0, help="kernel selector passed to lordba_forward_algo (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the streaming reference kernel and the extra repetitions")
    ap.add_argument("--mode", choices=["forward", "stream", "copy"], default="forward",
                    help="forward: the adapter kernel (default).  stream / copy: run ONLY the streaming reference kernel "
                         "(read x, read y_base, write y_out) or a plain copy of x's bytes, for scaling profiler counters")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (token rows shard over GPUs with no exchange). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_24058_amd import binding, inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    binding.load_library()      # raises if the HIP library is missing: there is no fallback path

    if args.workload == "c5_model":
        args.steps = 10 if args.steps is None else args.steps
        args.warmup = 1 if args.warmup is None else args.warmup
        return bench_c5_model(args)
    if args.ptq:
        args.steps = 20 if args.steps is None else args.steps
        args.warmup = 3 if args.warmup is None else args.warmup
        return bench_ptq(args)
    args.steps = 2400 if args.steps is None else args.steps
    args.warmup = 240 if args.warmup is None else args.warmup
    if args.workload == "c4_sweep":
        return bench_c4_sweep(args)
    if args.backward or args.train_step:
        args.steps = min(args.steps, 600)
        return bench_backward(args)
    sh = _shape(args.workload)

    # ---- inputs: one adapter, `sets` activation sets, all resident in HBM before timing ------------------------
    per_set = sh.activation_bytes()
    sets = args.sets if args.sets > 0 else max(2, -(-2 * CACHE_BYTES // per_set) + 1)
    sets = min(sets, max(1, int(200e9 // per_set)))
    ell = args.ell
    nad = args.adapters
    host0 = inputs.make_inputs_for(sh, args.seed)
    if ell > 1:
        host0.update(inputs.make_envelopes(args.seed, sh.d_in, sh.d_out, sh.r, ell))
    if nad:
        host0.update(inputs.make_adapter_pool(args.seed, sh.d_in, sh.d_out, sh.r, nad) if ell == 1 else
                     inputs.make_adapter_pool_multi(args.seed, sh.d_in, sh.d_out, sh.r, nad, ell))
        host0["ids"] = inputs.make_adapter_ids(args.seed, sh.T, nad, args.id_pattern)
        pA, pB = binding.lordba_pack_pool(host0["signsA"], host0["signsB"])
    else:
        pA, pB = binding.lordba_pack_signs(host0["signsA"], host0["signsB"])
    dev = {k: torch.from_numpy(host0[k]).cuda() for k in ("s_in", "s_rank", "s_out")}
    if nad:
        dev["ids"] = torch.from_numpy(host0["ids"]).cuda()
    dev["packedA"] = torch.from_numpy(pA.view(np.int32)).cuda()
    dev["packedB"] = torch.from_numpy(pB.view(np.int32)).cuda()
    xs, ybs, youts = [], [], []
    for s in range(sets):
        act = host0 if s == 0 else inputs.make_activations(args.seed + 1000 * s, sh.T, sh.d_in, sh.d_out)
        xs.append(torch.from_numpy(act["x"]).cuda())
        ybs.append(torch.from_numpy(act["y_base"]).cuda())
        youts.append(torch.empty_like(ybs[-1]))
    torch.cuda.synchronize()

    ref = binding.load_bench_library() if (args.mode != "forward" or not args.no_ceiling) else None
    cur = lambda: torch.cuda.current_stream().cuda_stream

    if nad:
        def fwd(x, pa, pb, si, sr, so, yb, check=False, **kw):
            if ell > 1:
                return binding.lordba_forward_batched_multi(x, pa, pb, si, sr, so, dev["ids"], yb, **kw)
            return binding.lordba_forward_batched(x, pa, pb, si, sr, so, dev["ids"], yb, check=check, **kw)
    else:
        fwd = binding.lordba_forward if ell == 1 else binding.lordba_forward_multi

    def forward_step(i):
        s = i % sets
        fwd(xs[s], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
            ybs[s], y_out=youts[s], algo=args.algo, check=False)

    def hot_step(i):         # one buffer set only: the streams stay in the Infinity Cache
        fwd(xs[0], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
            ybs[0], y_out=youts[0], algo=args.algo, check=False)

    def stream_step(i):      # same buffers, same byte split, no arithmetic: the practical HBM ceiling
        s = i % sets
        rc = ref.lordba_bench_stream(xs[s].data_ptr(), ybs[s].data_ptr(), youts[s].data_ptr(),
                                     xs[s].numel() * 2, ybs[s].numel() * 2, cur())
        assert rc == 0, rc

    def copy_step(i):        # plain copy of known size (x's bytes into y_out's buffer if it fits, else into x of the next set)
        s = i % sets
        n = min(xs[s].numel(), youts[s].numel()) * 2
        rc = ref.lordba_bench_copy(xs[s].data_ptr(), youts[s].data_ptr(), n - n % 16, cur())
        assert rc == 0, rc

    step = {"forward": forward_step, "stream": stream_step, "copy": copy_step}[args.mode]

    K, W = args.steps, args.warmup
    use_graph = not args.no_graph
    full = args.mode == "forward" and not args.no_ceiling
    # The timed region of K steps is run REPS times after a warm-up of at least max(W, sets) steps and WARM_SECONDS of
    # untimed replays; the headline (value, ms_per_step, roofline) is the median repetition, all of them are listed.
    reps_us, walls = timed(step, K, max(W, sets), use_graph, reps=REPS)
    mid = _median_index(reps_us)
    kern_us = reps_us[mid]   # average launch-to-launch duration on the stream over that repetition's K steps
    wall_s = walls[mid]
    ms_per_step = wall_s * 1e3 / K
    alg_bytes = sh.algorithmic_bytes_multi(ell)
    if nad:                  # every adapter that some row uses is read once, plus the index array
        used = len(set(int(a) for a in host0["ids"] if 0 <= a < nad))
        alg_bytes = sh.activation_bytes() + used * (sh.adapter_bytes() + 2 * (ell - 1) * (sh.d_in + sh.r + sh.d_out)) + 4 * sh.T
    achieved = alg_bytes / (kern_us * 1e-6) / 1e9
    from paper_2605_24058_amd import traffic_profile
    traffic, traffic_note = traffic_profile.lookup("lordba_forward", sh.name) \
        if args.mode == "forward" and args.algo == 0 and ell == 1 and not nad else (None, "not measured for this mode")

    out = {
        "metric": "multi-adapter batch: adapter-branch tokens/s and achieved HBM GB/s" if nad else
                  "adapter-branch tokens/s and achieved HBM GB/s at d=4096, r=16, T=2048" if ell == 1 else
                  "multi-envelope adapter-branch tokens/s and achieved HBM GB/s",
        "value": sh.T * K / wall_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "io_dtype": "f16", "data": "synthetic",
        "config": {"workload": sh.name, "T": sh.T, "d_in": sh.d_in, "d_out": sh.d_out, "r": sh.r,
                   "ell": ell, "adapters": nad, "id_pattern": args.id_pattern if nad else None, "buffer_sets": sets, "launch": "hip_graph" if use_graph else "eager", "algo": args.algo,
                   "seed": args.seed, "mode": args.mode},
        "achieved_hbm_gbs": achieved, "hbm_peak_gbs": HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_note,
                     "kernel_us": kern_us, "algorithmic_bytes": alg_bytes,
                     "kernel_us_repetitions": reps_us, "statistic": "median of %d repetitions of the %d-step region" % (REPS, K)},
    }

    if full:
        c_us, _ = timed(stream_step, max(200, K // 4), 20, use_graph, reps=3)
        c_us = _median(c_us)
        h_us, _ = timed(hot_step, max(200, K // 4), 20, use_graph, reps=3)
        h_us = _median(h_us)
        forward_step(0)          # y_out of set 0 was overwritten by the reference kernel: restore it for the parity check
        torch.cuda.synchronize()
        out["stream_ceiling"] = {"what": "nontemporal read x + read y_base + write y_out, no arithmetic, same buffers",
                                 "kernel_us": c_us, "gbs": sh.activation_bytes() / (c_us * 1e-6) / 1e9,
                                 "forward_vs_ceiling": c_us / kern_us}
        out["cache_resident"] = {"what": "same call on ONE buffer set (streams served by the 256 MB Infinity Cache): not HBM",
                                 "kernel_us": h_us, "gbs": alg_bytes / (h_us * 1e-6) / 1e9}

    # ---- CPU baseline: the fp64 oracle as it stands, on the host cores, same workload (bounded sample) ---------
    if not args.no_cpu_baseline and args.mode == "forward":
        import oracle
        cores = oracle.available_cores()
        budget_macs = 4e9                        # keeps the leg to a few seconds at ~1e9 fp64 MAC/s/core
        macs = sh.sign_macs() * ell * (8 if nad else 1)      # the batched oracle runs on one thread
        rows = sh.T if macs <= budget_macs else max(16, int(sh.T * budget_macs / macs))
        idx = np.arange(rows) if rows == sh.T else np.linspace(0, sh.T - 1, rows).astype(np.int64)
        xh, ybh = host0["x"][idx], host0["y_base"][idx]
        ofwd = oracle.forward if ell == 1 else oracle.forward_multi
        if nad:              # the batched oracle is single-threaded: the thread count is ignored
            ids_h = host0["ids"][idx]
            obatched = oracle.forward_batched if ell == 1 else oracle.forward_batched_multi
            ofwd = lambda x, sa, sb, si, sr, so, yb, nthreads=1: obatched(
                x, sa, sb, si, sr, so, ids_h[:x.shape[0]], yb)
            cores = 1
        run = lambda nt: ofwd(xh, host0["signsA"], host0["signsB"], host0["s_in"], host0["s_rank"],
                              host0["s_out"], ybh, nthreads=nt)
        c0 = time.perf_counter(); want = run(cores); c1 = time.perf_counter()
        s_rows = max(1, rows // 8)
        c2 = time.perf_counter()
        ofwd(xh[:s_rows], host0["signsA"], host0["signsB"], host0["s_in"], host0["s_rank"], host0["s_out"],
             ybh[:s_rows], nthreads=1)
        c3 = time.perf_counter()
        got = youts[0].cpu().numpy()[idx].astype(np.float64)
        err = float(oracle.row_rel_l2(got, want).max())
        out["cpu_baseline"] = {"value": rows / (c1 - c0), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": "%d of %d token rows of the same workload, all %d host threads" % (rows, sh.T, cores),
                               "single_thread_tokens_per_s": s_rows / (c3 - c2),
                               "gbs_equiv": rows / sh.T * alg_bytes / (c1 - c0) / 1e9}
        out["parity_max_row_rel_l2"] = err
        out["parity_ok"] = bool(err <= 1e-3)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
