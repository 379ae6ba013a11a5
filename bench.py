#!/usr/bin/env python3
"""ISOPO layer-step benchmark on one MI355X.

A step is one pass of the whole hot path over one transformer block's seven
linear projections: isopo_layer_gram per projection (per-sequence gradients to
that projection's stash + their Gram matrix K)  ->  ONE batched isopo_transform
for the block's seven Gram matrices (interacting coefficients)  ->
isopo_weighted_grad per projection (dW from the stash).  Inputs are synthetic,
seeded, and resident in HBM before the timed region starts.

Prints ONE JSON line: tokens/s for the block step, TFLOP/s on algorithmic
FLOPs, the dominant kernel's roofline (live HIP-event timing), the overhead
over the plain REINFORCE contraction, and the CPU oracle timed on a bounded
sample of the same workload.  "variants" holds the same block timed for the
other routes to the coefficients (Fisher norms from K; Fisher norms from
token-position samples followed by one weighted contraction), each with its
overhead over REINFORCE.  --config config4 sweeps the 28-layer stack and adds
the lambda sweep for both variants under "sweep".
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

PEAK_BF16_MFMA = 2.5e15     # MI355X dense bf16 matrix peak, flop/s
PEAK_HBM = 8.0e12           # B/s


def algorithmic_flops(n_tokens: int, d_in: int, d_out: int, n_seq: int) -> dict:
    D = d_in * d_out
    return {"seq_grads": 2.0 * n_tokens * D, "gram": float(n_seq * (n_seq + 1)) * D,
            "weighted": 2.0 * n_seq * D, "solve": n_seq ** 3 / 3.0}


def read_traffic(kernel_tag: str):
    """HBM bytes per launch of the dominant kernel, from the committed counter summary."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def clock_dependence(args, block, layers, stash_views, fl, stream, wg_queue):
    """The same launch of the largest projection on all-zero operands.  The kernel executes the same
    instructions and cycles whatever the values; the part's power management does not: with operands
    that do not toggle it holds the full clock.  The ratio says how much of the gap to the 2.4 GHz
    peak is the clock under real data rather than the kernel's schedule."""
    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo
    big = max(range(len(block)), key=lambda i: layers[i].d_in * layers[i].d_out)
    lb = layers[big]
    X0, D0 = torch.zeros_like(lb.X), torch.zeros_like(lb.Delta)
    lz = isopo.Layer(X0, D0, block[big].seq_offsets)

    def time_launches(layer, n):
        ev = []
        for _ in range(n + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            isopo.seq_grads(layer, stash_views[big], stream=stream, max_workgroups=256, queue=wg_queue,
                            layout=isopo.stash_layout(layer)[0])
            e1.record(stream)
            ev.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in ev[1:]])) * 1e-3

    t_zero, t_real = time_launches(lz, 4), time_launches(lb, 4)
    power = None
    if args.board_probe:
        # what the board reports while each case runs for a few seconds: socket power and the XCDs' clocks
        import re
        import subprocess
        import threading

        def smi():
            try:
                out = subprocess.run(["amd-smi", "metric", "-p", "-c"], capture_output=True, text=True, timeout=20).stdout
            except (OSError, subprocess.SubprocessError):
                return None
            pw = re.search(r"SOCKET_POWER:\s*(\d+)", out)
            clk = [int(x) for x in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)", out)]
            return {"socket_power_w": int(pw.group(1)) if pw else None, "xcd_clocks_mhz": clk[:8]}

        def sustained(layer, seconds=4.0):
            stop = time.time() + seconds
            samples = []

            def poll():
                time.sleep(1.5)
                while time.time() < stop - 0.3:
                    samples.append(smi())
                    time.sleep(0.7)
            th = threading.Thread(target=poll)
            th.start()
            while time.time() < stop:
                for _ in range(20):
                    isopo.seq_grads(layer, stash_views[big], stream=stream, max_workgroups=256, queue=wg_queue,
                            layout=isopo.stash_layout(layer)[0])
                torch.cuda.synchronize()
            th.join()
            return [x for x in samples if x]
        power = {"zero_operands": sustained(lz), "workload": sustained(lb)}
    return {"projection": block[big].name, **({"board": power} if power else {}), "tflops_on_the_workload": fl[big]["seq_grads"] / t_real / 1e12,
            "tflops_on_zero_operands": fl[big]["seq_grads"] / t_zero / 1e12,
            "zero_ms": t_zero * 1e3, "workload_ms": t_real * 1e3,
            "what": "same launch, same cycles; the clock under random operands is 1.85 - 2.0 GHz, on zeros 2.4 GHz (profiles/)"}


def mfma_ceiling(dev, board_probe=False) -> dict:
    """What the matrix cores sustain on this board when they do nothing else: isopo_probe_mfma_loop (one wave
    per SIMD, 256 accumulator registers, operands in registers, no memory traffic in the loop) for the two bf16
    MFMA shapes, on random operands (sign, mantissa and a few exponents random: every operand bit toggles) and on
    zeros.  The rate on random operands is the ceiling a contraction of this register shape can reach under the
    board's power limit; the rate on zeros shows the clock the part holds when the operands do not toggle."""
    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo
    stream = torch.cuda.current_stream()
    n_words = isopo.PROBE_THREADS * 64                       # 16 vectors of four 32-bit words per thread
    g = torch.Generator(device="cpu").manual_seed(7)

    def half_words():
        sign = torch.randint(0, 2, (n_words,), generator=g, dtype=torch.int32) << 15
        expo = (0x7e + torch.randint(0, 3, (n_words,), generator=g, dtype=torch.int32)) << 7    # values near 1
        mant = torch.randint(0, 128, (n_words,), generator=g, dtype=torch.int32)
        return sign | expo | mant
    rand_ops = (half_words() | (half_words() << 16)).to(dev)
    zero_ops = torch.zeros_like(rand_ops)
    sink = torch.empty(isopo.PROBE_THREADS, dtype=torch.float32, device=dev)
    iters = 20000
    flops = 2.0 * 128 * 128 * 32 * iters * (isopo.PROBE_THREADS // 64)
    out = {"what": "loop of bf16 MFMAs only: 256 workgroups x 4 waves, 256 accumulator registers per lane, operands in "
                   "registers; TFLOP/s sustained over launches of about 40 ms", "iters_per_launch": iters, "rates": {}}
    for shape, name in ((32, "v_mfma_f32_32x32x16_bf16"), (16, "v_mfma_f32_16x16x32_bf16")):
        for ops, kind in ((rand_ops, "random_operands"), (zero_ops, "zero_operands")):
            ms = []
            for rep in range(6):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                isopo.probe_mfma_loop(shape, ops, sink, iters, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1))
            t = float(np.median(ms[1:])) * 1e-3
            out["rates"][f"{name}/{kind}"] = {"tflops": flops / t / 1e12, "ms": t * 1e3,
                                               "frac_of_2.5_pflops": flops / t / PEAK_BF16_MFMA}
    return out


def schedule_probe(dev) -> dict:
    """Is the contraction bound by its schedule or by the board?  (1) isopo_probe_lds_dma: the rate at which a
    workgroup streams an L2-resident buffer into LDS with the contraction's DMA loads, against the number of waves
    that issue them; (2) isopo_probe_contraction_waves: config 3's gate projection (dW = Delta^T X, 256x256 tiles)
    with 4 waves per workgroup (the per-sequence launch's shape) and with 8 (what the sums over all tokens launch:
    half the registers per wave, twice the DMA issuers), on the workload's operands and on zeros (where the part
    holds its top clock)."""
    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo, workloads as wl
    stream = torch.cuda.current_stream()

    def med_ms(fn, reps=7):
        ms = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        return float(np.median(ms[1:]))
    out = {"lds_dma": {"what": "GB/s per workgroup into LDS, ring of 32 KiB stages refilled without a pause, 16 MiB "
                               "buffer (L2-resident); 8 workgroups (alone on the chip) and 256 (one per compute unit)",
                       "rates": {}},
           "contraction": {"what": "config3 gate projection, dW = Delta^T X, ms per launch and TFLOP/s on 2 N d_out d_in flop"}}
    buf = torch.ones(16 << 20, dtype=torch.uint8, device=dev)
    sink = torch.empty(4096, dtype=torch.float32, device=dev)
    iters = 4000
    for wgs in (8, 256):
        for waves in (2, 4, 8, 16):
            for stages in (2, 4):
                t = med_ms(lambda: isopo.probe_lds_dma(buf, waves, stages, wgs, iters, sink, stream=stream), reps=4)
                out["lds_dma"]["rates"][f"{wgs}_workgroups/{waves}_waves/{stages}_stages"] = round(iters * 32768 / t / 1e6, 1)
    w = wl.CONFIGS["config3"]
    lengths = wl.draw_lengths(w)
    gate = [p for p in w.projections if p.name == "gate"][0]
    prob = wl.make_layer(w, gate, lengths, device=dev)
    flops = 2.0 * prob.n_tokens * prob.d_in * prob.d_out
    zX, zD = torch.zeros_like(prob.X), torch.zeros_like(prob.Delta)
    dW = torch.empty((prob.d_out, prob.d_in), dtype=torch.float32, device=dev)
    for kind, layer in (("workload", isopo.Layer(prob.X, prob.Delta, prob.seq_offsets)),
                        ("zero_operands", isopo.Layer(zX, zD, prob.seq_offsets))):
        for waves in (4, 8, 4, 8):
            t = med_ms(lambda: isopo.probe_contraction_waves(layer, waves, dW, stream=stream), reps=9)
            out["contraction"].setdefault(f"{kind}/{waves}_waves", []).append({"ms": round(t, 4), "tflops": round(flops / t / 1e9, 1)})
    return out


def ghost_case(dev) -> dict:
    """The ghost Gram path where it is the chosen one: a short microbatch (8 sequences of 1024 tokens) on the
    stress layer 5120 -> 27648.  Algorithmic work N^2 (d_in + d_out) flop (both token-by-token products over the
    pairs t <= s)."""
    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo, workloads as wl
    stream = torch.cuda.current_stream()
    w = wl.CONFIGS["config5"]
    prob = wl.make_layer(w, w.projections[0], np.full(8, 1024, dtype=np.int64), device=dev)
    layer = isopo.Layer(prob.X, prob.Delta, prob.seq_offsets)
    chosen, full, _ = isopo.gram_plan(layer, "auto")
    ws = isopo.alloc_workspace(isopo.gram_plan(layer, "ghost")[1], dev)
    K = torch.empty((prob.n_seq, prob.n_seq), dtype=torch.float32, device=dev)
    ms = []
    for _ in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        isopo.layer_gram(layer, "ghost", K=K, workspace=ws, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    t = float(np.median(ms[2:])) * 1e-3
    flops = float(prob.n_tokens) ** 2 * (prob.d_in + prob.d_out)
    return {"workload": f"ghost Gram, {prob.d_in}x{prob.d_out}, {prob.n_seq} sequences, N={prob.n_tokens} tokens, bf16",
            "auto_choice": chosen, "ms": t * 1e3, "tflops": flops / t / 1e12, "frac_of_bf16_peak": flops / t / PEAK_BF16_MFMA,
            "what": "isopo_layer_gram(path = GHOST): fill, token -> sequence map, ghost_gram_tiled_kernel, finish"}


def eigh_case(dev) -> dict:
    """The eigendecomposition route against the Cholesky transform it competes with: one Gram matrix of B
    sequences (a spread spectrum, as Gram matrices of gradients have), D, U = eigh(K) once, then the sweep of three
    regularisers from it; beside it three Cholesky transforms.  Both routes at every B on the same matrix."""
    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo
    stream = torch.cuda.current_stream()
    lambdas = [1e-4, 1e-3, 1e-2]
    out = {"what": "isopo_ntk_eigh + isopo_transform_eigh(3 lambdas) against 3 x isopo_transform(INTERACTING); ms, "
                   "median of 5 after one warm-up", "sizes": {}}
    for m in (32, 64, 94, 96, 128, 200, 256, 512):
        rng = np.random.default_rng(m)
        J = rng.standard_normal((m, 4 * m)) * np.logspace(0, -2, 4 * m)[None, :]
        K = torch.from_numpy((J @ J.T).astype(np.float32)).to(dev)
        A = torch.from_numpy(rng.standard_normal(m).astype(np.float32)).to(dev)
        ws = isopo.alloc_workspace(isopo.load().isopo_ntk_eigh_workspace(m, 1), dev)
        tws = isopo.alloc_workspace(max(isopo.transform_workspace(m, 1), 256), dev)

        def med(fn):
            ms = []
            for _ in range(6):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                fn()
                e1.record(stream)
                torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1))
            return float(np.median(ms[1:]))
        D, U, info = isopo.ntk_eigh(K, workspace=ws)
        t_eigh = med(lambda: isopo.ntk_eigh(K, workspace=ws))
        t_sweep = med(lambda: isopo.transform_eigh(D, U, A, lambdas, isopo.REG_REL_TRACE))
        t_chol = med(lambda: [isopo.transform(K, A, "interacting", lam, isopo.REG_REL_TRACE, workspace=tws) for lam in lambdas])
        out["sizes"][str(m)] = {"eigh_ms": t_eigh, "sweep_of_3_from_eigh_ms": t_sweep, "three_cholesky_transforms_ms": t_chol,
                                "route": "jacobi" if m <= 94 else "tridiagonal + QL", "info": int(info.item())}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--no-clock-dependence", action="store_true",
                    help="skip the zero-operand launches of the largest projection (keeps kernel profiles to the step's own launches)")
    ap.add_argument("--board-probe", action="store_true",
                    help="with --clock-probe: also sample socket power and XCD clocks (amd-smi, a child process) while "
                         "each case loops for four seconds; not under rocprofv3, whose preloaded library makes every "
                         "child a GPU process")
    ap.add_argument("--clock-probe", action="store_true",
                    help="only time the largest projection's stash launch on zero operands and on the workload, then exit")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="only time a loop of nothing but bf16 MFMAs (both shapes, random and zero operands, the "
                         "contraction's register shape) and print the sustained rates, then exit")
    ap.add_argument("--ghost-case", action="store_true",
                    help="only time isopo_layer_gram on the ghost path for a short microbatch on the stress layer "
                         "(5120 -> 27648, 8 sequences of 1024 tokens) and print its rate, then exit")
    ap.add_argument("--schedule-probe", action="store_true",
                    help="only run the two schedule diagnostics (LDS-DMA rate against waves per workgroup; the gate "
                         "projection's contraction with 4 and with 8 waves, on the workload and on zeros), then exit")
    ap.add_argument("--eigh-case", action="store_true",
                    help="only time the eigendecomposition route (decomposition, sweep of three regularisers) against "
                         "three Cholesky transforms for 32 to 512 sequences, then exit")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="config3", choices=["config2", "config3", "config4", "config5"])
    ap.add_argument("--variant", default="interacting", choices=["fisher", "interacting"])
    ap.add_argument("--lam", type=float, default=1e-3)
    ap.add_argument("--n-samples", type=int, default=32, help="token-position samples of the Fisher estimate")
    ap.add_argument("--no-variants", action="store_true", help="time the headline route only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true", help="skip the torch.matmul context timing")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (untimed): the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer step has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2512_23353_amd import isopo, workloads as wl

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.mfma_ceiling:
        print(json.dumps(mfma_ceiling(dev, args.board_probe)))
        return 0
    if args.eigh_case:
        print(json.dumps(eigh_case(dev)))
        return 0
    if args.schedule_probe:
        print(json.dumps(schedule_probe(dev)))
        return 0
    if args.ghost_case:
        print(json.dumps(ghost_case(dev)))
        return 0
    w = wl.CONFIGS[args.config]
    lengths = wl.draw_lengths(w)
    # a multi-layer stack is swept layer by layer; two distinct layers' inputs alternate (28 would not fit HBM)
    n_layers = w.n_layers
    blocks = [wl.make_block(w, device=dev, lengths=lengths, layer=l) for l in range(min(n_layers, 2))]
    block = [p for b in blocks for p in b]
    n_tokens, n_seq = block[0].n_tokens, block[0].n_seq
    layers = [isopo.Layer(p.X, p.Delta, p.seq_offsets) for p in block[:1]]
    layers += [isopo.Layer(p.X, p.Delta, p.seq_offsets, seq_offsets_dev=layers[0].off_dev) for p in block[1:]]
    sweeps = n_layers // len(blocks)          # passes over `layers` per step
    assert sweeps * len(blocks) == n_layers
    A = torch.from_numpy(block[0].A).to(dev)
    plans = [isopo.gram_plan(l) for l in layers]
    npj = len(blocks[0])                      # projections per block
    # One workspace (stash + Gram partials) per projection of a block, so that the block's seven Gram
    # matrices exist together and ONE batched transform launch solves all seven problems.
    wss = [isopo.alloc_workspace(max(plans[b * npj + j][1] for b in range(len(blocks))), dev) for j in range(npj)]
    ws = wss[max(range(npj), key=lambda j: wss[j].numel())]
    Kb = [torch.empty((npj, n_seq, n_seq), dtype=torch.float32, device=dev) for _ in blocks]
    cb = [torch.empty((npj, n_seq), dtype=torch.float32, device=dev) for _ in blocks]
    infob = [torch.zeros(npj, dtype=torch.int32, device=dev) for _ in blocks]
    Ab = torch.from_numpy(block[0].A).to(dev).repeat(npj, 1).contiguous()
    Ks = [Kb[i // npj][i % npj] for i in range(len(layers))]
    cs = [cb[i // npj][i % npj] for i in range(len(layers))]
    infos = [infob[i // npj][i % npj: i % npj + 1] for i in range(len(layers))]
    dWs = [torch.zeros((l.d_out, l.d_in), dtype=torch.float32, device=dev) for l in layers]
    tws = isopo.alloc_workspace(isopo.transform_workspace(n_seq, npj), dev)
    stream = torch.cuda.current_stream()
    assert all(pl[0] == "materialised" for pl in plans), "the benchmark shapes all take the materialised path"

    # the kept stash in the layout the library prefers for each layer (tile order for these shapes)
    layouts = [isopo.stash_layout(l)[0] for l in layers]

    def make_step(variant, lam):
        def step():
            for _ in range(sweeps):
                for b in range(len(blocks)):
                    for j in range(npj):
                        isopo.layer_gram(layers[b * npj + j], "auto", K=Kb[b][j], workspace=wss[j],
                                         keep_stash=isopo.KEEP_FAST, stream=stream)
                    isopo.transform(Kb[b], Ab, variant, lam, isopo.REG_REL_TRACE, c=cb[b], info=infob[b], workspace=tws,
                                    stream=stream)
                    for j in range(npj):
                        isopo.weighted_grad(layers[b * npj + j], cb[b][j], wss[j], 0.0, dWs[b * npj + j], stream=stream,
                                            layout=layouts[b * npj + j])
        return step

    step = make_step(args.variant, args.lam)

    def reinforce_step():
        for _ in range(sweeps):
            for l, dW in zip(layers, dWs):
                isopo.weighted_grad(l, None, None, 0.0, dW, stream=stream)

    # Non-interacting update with the token-position-sample Fisher estimate: coefficients first, then ONE
    # weighted contraction (rows of the narrower operand pre-scaled).  No stash, no Gram matrix.
    g = torch.Generator(device="cpu").manual_seed(w.seed)
    sample_idx = torch.randperm(n_tokens, generator=g)[: args.n_samples].to(torch.int32).to(dev)
    # projections that share their input (q/k/v, gate/up) form one group: X is streamed once per group
    groups = []
    for i, l in enumerate(layers):
        same_block = groups and groups[-1][0] // npj == i // npj
        if same_block and len(groups[-1]) < 4 and layers[groups[-1][0]].X.data_ptr() == l.X.data_ptr():
            groups[-1].append(i)
        else:
            groups.append([i])
    fs_ws = isopo.alloc_workspace(max(isopo.load().isopo_fisher_samples_group_workspace(layers[g[0]].ref(), len(g),
                                                                                        args.n_samples)
                                      for g in groups), dev)
    f2b = [torch.empty((npj, n_seq), dtype=torch.float32, device=dev) for _ in blocks]

    def token_sample_step_group_calls():
        for _ in range(sweeps):
            for g in groups:
                b, j0 = g[0] // npj, g[0] % npj
                isopo.fisher_samples_group([layers[i] for i in g], sample_idx, A, args.lam, isopo.REG_REL_TRACE,
                                           cb[b][j0:j0 + len(g)], f2b[b][j0:j0 + len(g)], fs_ws, stream=stream)
                for i in g:
                    isopo.weighted_grad(layers[i], cs[i], None, 0.0, dWs[i], stream=stream)

    # A block's groups in one launch (isopo_fisher_samples_block): their workgroups fill the chip one group after
    # the other, and only the last group's last round leaves compute units idle.
    block_groups = [[[layers[i] for i in g] for g in groups if g[0] // npj == b] for b in range(len(blocks))]
    fsb_ws = isopo.alloc_workspace(isopo.load().isopo_fisher_samples_block_workspace(layers[0].ref(), npj, args.n_samples), dev)

    def token_sample_step():
        for _ in range(sweeps):
            for b in range(len(blocks)):
                isopo.fisher_samples_block(block_groups[b], sample_idx, A, args.lam, isopo.REG_REL_TRACE, cb[b], f2b[b],
                                           fsb_ws, stream=stream)
                for j in range(npj):
                    i = b * npj + j
                    isopo.weighted_grad(layers[i], cs[i], None, 0.0, dWs[i], stream=stream)

    # The same with the Fisher passes of a block's groups on streams of their own (default priority): they are
    # independent of one another, and run side by side the nearly empty last round of one launch's workgroups
    # (a quarter of a launch at this size) overlaps the others' main rounds.  The contractions follow on the
    # launch stream once all coefficients are there.
    n_side = max(len([g for g in groups if g[0] // npj == b]) for b in range(len(blocks)))
    side = [torch.cuda.Stream(device=dev) for _ in range(n_side)]
    fs_wss = [isopo.alloc_workspace(fs_ws.numel(), dev) for _ in range(n_side)]
    ev_go = torch.cuda.Event()
    ev_done = [torch.cuda.Event() for _ in range(n_side)]

    def token_sample_step_side_streams():
        for _ in range(sweeps):
            for b in range(len(blocks)):
                mine = [g for g in groups if g[0] // npj == b]
                ev_go.record(stream)
                for k, g in enumerate(mine):
                    j0 = g[0] % npj
                    side[k].wait_event(ev_go)
                    isopo.fisher_samples_group([layers[i] for i in g], sample_idx, A, args.lam, isopo.REG_REL_TRACE,
                                               cb[b][j0:j0 + len(g)], f2b[b][j0:j0 + len(g)], fs_wss[k], stream=side[k])
                    ev_done[k].record(side[k])
                for k in range(len(mine)):
                    stream.wait_event(ev_done[k])
                for g in mine:
                    for i in g:
                        isopo.weighted_grad(layers[i], cs[i], None, 0.0, dWs[i], stream=stream)

    medians = {}

    def timed(fn, steps, warmup, tag=None):
        """Seconds per step: wall clock over exactly `steps` steps between two device synchronisations.
        Every step is also bracketed by HIP events on the launch stream; their median goes to medians[tag]."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for e0, e1 in ev:
            e0.record(stream)
            fn()
            e1.record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        if tag is not None:
            medians[tag] = float(np.median([a.elapsed_time(b) for a, b in ev]))
        return wall

    t_step = timed(step, args.steps, args.warmup, "step")
    assert all(int(i.sum().item()) == 0 for i in infob), "transform reported a non-positive pivot"
    t_reinforce = timed(reinforce_step, max(3, args.steps // 2), 2, "reinforce")

    # Dominant kernel: the per-sequence gradient contraction, one launch per projection.
    # Average launch duration over the block's seven launches, HIP events on the launch stream.
    stash_views = [ws[: isopo.stash_nbytes(l)].view(torch.bfloat16 if l.dtype == isopo.BF16 else torch.float32)
                   .view(l.n_seq, l.d_out, l.d_in) for l in layers]
    reps = max(3, args.steps // 2)
    wg_queue = torch.zeros(8, dtype=torch.int32, device=dev)
    durs = []
    for _ in range(reps):
        for l, sv in zip(layers, stash_views):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            # the launch isopo_layer_gram makes: one persistent workgroup per compute unit
            isopo.seq_grads(l, sv, stream=stream, max_workgroups=256, queue=wg_queue, layout=isopo.stash_layout(l)[0])
            e1.record(stream)
            durs.append((e0, e1))
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in durs][len(layers):] or [a.elapsed_time(b) for a, b in durs]
    avg_launch_s = float(np.mean(ms)) * 1e-3
    fl = [algorithmic_flops(n_tokens, l.d_in, l.d_out, n_seq) for l in layers]
    seq_grad_flops_per_launch = float(np.mean([f["seq_grads"] for f in fl]))

    # The same launch of the largest projection on all-zero operands.  The kernel executes the same
    # instructions and cycles whatever the values; the part's power management does not: with operands
    # that do not toggle it holds the full clock.  The ratio says how much of the gap to the 2.4 GHz
    # peak is the clock under real data rather than the kernel's schedule.
    zero_operands = None
    if not args.no_clock_dependence or args.clock_probe:
        zero_operands = clock_dependence(args, block, layers, stash_views, fl, stream, wg_queue)
        if args.clock_probe:
            # for a counter run (GRBM_GUI_ACTIVE): five launches on zeros, then five on the workload, nothing else
            # after; no child processes unless --board-probe asks for them
            print(json.dumps({k: zero_operands[k] for k in ("projection", "zero_ms", "workload_ms", "board") if k in zero_operands}))
            return 0
    total_flops = float(sum(sum(f.values()) for f in fl)) * sweeps
    reinforce_flops = float(sum(f["seq_grads"] for f in fl)) * sweeps
    stash_bytes_per_step = float(sum(2.0 * n_seq * l.d_in * l.d_out for l in layers)) * sweeps

    variants, sweep_report = {}, None
    if not args.no_variants:
        reps = max(2, args.steps // 3)
        other = "fisher" if args.variant == "interacting" else "interacting"
        t_other = timed(make_step(other, args.lam), reps, 2, "other")
        t_ts = timed(token_sample_step, reps, 2, "token_samples")
        t_tsg = timed(token_sample_step_group_calls, reps, 2, "token_samples_groups")
        t_ts2 = timed(token_sample_step_side_streams, reps, 2, "token_samples_side")

        dWs_bf16 = [torch.zeros(dW.shape, dtype=torch.bfloat16, device=dev) for dW in dWs]

        def variant_step(reg_mode=isopo.REG_REL_TRACE, beta=0.0, recompute=False, bf16_dw=False):
            def fn():
                for _ in range(sweeps):
                    for b in range(len(blocks)):
                        for j in range(npj):
                            isopo.layer_gram(layers[b * npj + j], "auto", K=Kb[b][j], workspace=wss[j],
                                             keep_stash=0 if recompute else isopo.KEEP_FAST, stream=stream)
                        isopo.transform(Kb[b], Ab, args.variant, args.lam, reg_mode, c=cb[b], info=infob[b], workspace=tws,
                                        stream=stream)
                        for j in range(npj):
                            i = b * npj + j
                            if recompute:
                                isopo.weighted_grad(layers[i], cb[b][j], None, beta, dWs[i], stream=stream)
                            elif bf16_dw:
                                isopo.weighted_grad_stash_bf16(layers[i], cb[b][j], wss[j], layouts[i], beta, dWs_bf16[i],
                                                               stream=stream)
                            else:
                                isopo.weighted_grad(layers[i], cb[b][j], wss[j], beta, dWs[i], stream=stream, layout=layouts[i])
            return fn
        t_abs = timed(variant_step(reg_mode=isopo.REG_ABSOLUTE), reps, 2, "absolute")
        t_beta = timed(variant_step(beta=1.0), reps, 2, "beta1")
        t_rec = timed(variant_step(recompute=True), reps, 2, "recompute")
        t_bf = timed(variant_step(bf16_dw=True), reps, 2, "bf16_dw")
        t_bf1 = timed(variant_step(beta=1.0, bf16_dw=True), reps, 2, "bf16_dw_beta1")
        del dWs_bf16
        # The headline step and the REINFORCE baseline replayed from HIP graphs: what the gaps between the step's
        # launches cost (the library allocates nothing and clears its counters with kernels, so a caller may
        # capture it).  One block only: the sweep of config 4 would be a graph of some thousand nodes.
        t_gs = t_gr = None
        graph_note = None
        if len(blocks) == 1 and sweeps == 1:
            outer = stream
            try:
                g_step, g_reinforce = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_step):
                    stream = torch.cuda.current_stream()       # the closures launch on the capturing stream
                    step()
                with torch.cuda.graph(g_reinforce):
                    stream = torch.cuda.current_stream()
                    reinforce_step()
                stream = outer
                t_gs = timed(g_step.replay, reps, 2, "graph_step")
                t_gr = timed(g_reinforce.replay, reps, 2, "graph_reinforce")
            except RuntimeError as e:                          # the variant is extra: the bench line does not depend on it
                stream = outer
                t_gs = t_gr = None
                graph_note = f"graph capture failed: {e}"
                torch.cuda.synchronize()
        for dW in dWs:
            dW.zero_()          # beta = 1 accumulated into them

        # algorithmic flops of the token-sample route: the contraction and the two token-by-sample products
        ts_flops = reinforce_flops + sweeps * 2.0 * n_tokens * args.n_samples * float(
            sum(layers[g[0]].d_in + sum(layers[i].d_out for i in g) for g in groups))

        def entry(t, tag, flops=None, **more):
            rate = {} if flops is None else {"tflops": flops / t / 1e12, "pct_bf16_mfma_peak": 100.0 * flops / t / PEAK_BF16_MFMA}
            return {"ms_per_step": t * 1e3, "ms_per_step_median_hip_events": medians.get(tag),
                    "overhead_over_reinforce": t / t_reinforce - 1.0, **rate, **more}
        variants = {
            f"{args.variant}_from_stash_gram": entry(t_step, "step", total_flops),
            f"{other}_from_stash_gram": entry(t_other, "other", total_flops),
            f"{args.variant}_absolute_lambda": entry(t_abs, "absolute", what="the headline route with reg = lambda as printed (numerically nil at these shapes: K_ii ~ 1e4..1e6)"),
            f"{args.variant}_beta_1": entry(t_beta, "beta1", what="the headline route accumulating into dW (mod.grad += of the listings): one more read of dW per projection"),
            f"{args.variant}_bf16_dW": entry(t_bf, "bf16_dw", what="the headline route with dW written in bf16 (isopo_weighted_grad_stash_bf16: the gradient buffer of a bf16 parameter); the REINFORCE baseline it is set against still writes fp32"),
            f"{args.variant}_bf16_dW_beta_1": entry(t_bf1, "bf16_dw_beta1", what="the same accumulating into the bf16 dW"),
            f"{args.variant}_without_stash": entry(t_rec, "recompute", what="isopo_layer_gram with no stash kept, then isopo_weighted_grad(c, stash = NULL): the weighted contraction from X and Delta again (the route for a workspace too small to keep the stash)"),
            "fisher_from_token_samples": entry(t_ts, "token_samples", ts_flops, n_samples=args.n_samples,
                                               what="isopo_fisher_samples_block once per block (the sets of projections sharing an input in one launch), then isopo_weighted_grad(c, stash = NULL) per projection: ONE weighted contraction, no stash, no scaled copy"),
            "fisher_from_token_samples_group_calls": entry(t_tsg, "token_samples_groups", ts_flops, n_samples=args.n_samples,
                                                           what="the same with one isopo_fisher_samples_group call per set of projections sharing an input"),
            "fisher_from_token_samples_side_streams": entry(t_ts2, "token_samples_side", ts_flops, n_samples=args.n_samples,
                                                            what="the group calls on streams of their own, side by side, before the contractions on the launch stream"),
        }
        if t_gs is not None:
            variants[f"{args.variant}_replayed_from_hip_graph"] = entry(
                t_gs, "graph_step", total_flops, reinforce_replayed_ms=t_gr * 1e3,
                overhead_over_replayed_reinforce=t_gs / t_gr - 1.0,
                what="the headline step and the REINFORCE baseline each captured once in a HIP graph and replayed: the same kernels without the host's launch gaps")
        elif graph_note is not None:
            variants[f"{args.variant}_replayed_from_hip_graph"] = {"note": graph_note}
        if n_layers > 1:
            # The sweep with K and the stash formed once per layer: six transforms (both variants x three
            # lambdas) and six stash-weighted sums per projection, against ONE REINFORCE sweep.
            lams = (1e-4, 1e-3, 1e-2)
            c6 = [[torch.empty(n_seq, dtype=torch.float32, device=dev) for _ in range(6)] for _ in layers]
            dW6 = [[torch.empty_like(dW) for _ in range(6)] for dW in dWs[: len(blocks[0])]]

            def shared_sweep_step():
                for _ in range(sweeps):
                    for li, (l, pl, K, info) in enumerate(zip(layers, plans, Ks, infos)):
                        assert pl[0] == "materialised"
                        wsl = wss[li % npj]
                        isopo.layer_gram(l, "auto", K=K, workspace=wsl, keep_stash=isopo.KEEP_FAST, stream=stream)
                        for vi, variant in enumerate(("fisher", "interacting")):
                            for k, lam in enumerate(lams):
                                isopo.transform(K, A, variant, lam, isopo.REG_REL_TRACE, c=c6[li][3 * vi + k], info=info,
                                                stream=stream)
                        for k in range(6):
                            isopo.weighted_grad(l, c6[li][k], wsl, 0.0, dW6[li % len(dW6)][k], stream=stream,
                                                layout=layouts[li])

            t_shared = timed(shared_sweep_step, 2, 1)
            variants["sweep_with_shared_gram"] = {
                "ms_per_sweep": t_shared * 1e3, "updates_per_projection": 6,
                "overhead_over_one_reinforce_sweep": t_shared / t_reinforce - 1.0,
                "what": "per projection: stash + Gram once, 6 transforms (fisher, interacting) x lambda in (1e-4, 1e-3, 1e-2), 6 stash-weighted sums"}
            del dW6
            sweep_report = []
            for variant in ("fisher", "interacting"):
                for lam in (1e-4, 1e-3, 1e-2):
                    t = timed(make_step(variant, lam), 2, 1)
                    assert all(int(i.sum().item()) == 0 for i in infob)
                    sweep_report.append({"variant": variant, "lambda": lam, "ms_per_sweep": t * 1e3,
                                         "overhead_over_reinforce": t / t_reinforce - 1.0})
    achieved = seq_grad_flops_per_launch / avg_launch_s

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    context = {}
    if not args.no_context:
        def torch_reinforce():
            for _ in range(sweeps):
                for p, dW in zip(block, dWs):
                    a_tok = torch.repeat_interleave(A, torch.from_numpy(np.diff(p.seq_offsets)).to(dev)).to(p.Delta.dtype)
                    torch.matmul((p.Delta * a_tok[:, None]).T, p.X, out=None)
        context["torch_matmul_reinforce_ms"] = timed(torch_reinforce, 3, 1) * 1e3

    out = {
        "metric": "ISOPO layer-step tokens/sec and TFLOP/s (% bf16 MFMA peak), 1 MI355X",
        "value": n_tokens / t_step, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "ms_per_step_median_hip_events": medians.get("step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {('one transformer block' if len(w.projections) > 1 else 'one layer') if n_layers == 1 else f'{n_layers} transformer blocks swept layer by layer'}, {len(w.projections)} projection{'s' if len(w.projections) > 1 else ''} "
                               f"({', '.join(f'{p.name} {p.d_in}x{p.d_out}' for p in w.projections)}), "
                               f"B={n_seq} ragged sequences, N={n_tokens} tokens, bf16 inputs fp32 accumulation",
                   "variant": args.variant, "lambda": args.lam, "reg_mode": "rel_trace",
                   "gram_paths": sorted(set(pl[0] for pl in plans)), "seed": w.seed},
        "device": {"name": torch.cuda.get_device_properties(dev).name,
                   "compute_units": torch.cuda.get_device_properties(dev).multi_processor_count,
                   "hbm_gib": round(torch.cuda.get_device_properties(dev).total_memory / 2 ** 30, 1),
                   "peaks_used": {"bf16_mfma_tflops": PEAK_BF16_MFMA / 1e12, "hbm_tb_s": PEAK_HBM / 1e12},
                   "clocks": "as found (not pinned); under the contraction the part runs at 1.85 - 2.0 GHz (board power cap) with the workload's random operands and at 2.4 GHz with zero operands, see profiles/"},
        "tflops": total_flops / t_step / 1e12,
        "pct_bf16_mfma_peak": 100.0 * total_flops / t_step / PEAK_BF16_MFMA,
        "algorithmic_flops_per_step": total_flops,
        "reinforce": {"ms_per_step": t_reinforce * 1e3, "ms_per_step_median_hip_events": medians.get("reinforce"), "tflops": reinforce_flops / t_reinforce / 1e12,
                      "overhead_of_isopo": t_step / t_reinforce - 1.0,
                      "overhead_floor_of_routes_through_K": stash_bytes_per_step * 2.0 / PEAK_HBM / t_reinforce,
                      "overhead_floor_what": "any route that forms K from a materialised stash reads the stash twice after the "
                                             "contraction that writes it (Gram pass, weighted sum): 2 x 2 B D bytes per "
                                             "projection at the 8 TB/s HBM peak, over this run's REINFORCE time; the write "
                                             "(issued under the MFMA-bound contraction) and everything else counted as free",
                      "what": "this library's own unweighted dW = Delta^T X over the same projections (advantages folded into Delta, as plain REINFORCE backprop does)", **context},
        "roofline": {"bound": "mfma", "kernel": "seq_grad_stream_kernel<256,256,4,1,true,true,true,false> (per-sequence gradients -> stash in tile order, persistent launch)",
                     "achieved": achieved / 1e12, "peak": PEAK_BF16_MFMA / 1e12, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_MFMA, "avg_launch_ms": avg_launch_s * 1e3,
                     "whole_step_frac": total_flops / t_step / PEAK_BF16_MFMA,
                     "note": "frac is the dominant kernel alone; whole_step_frac is the step's algorithmic flops over its time (pct_bf16_mfma_peak / 100)",
                     "flops_per_launch": seq_grad_flops_per_launch,
                     "traffic": read_traffic(f"seq_grad_{args.config}"),
                     **({"clock_dependence": zero_operands} if zero_operands else {})},
    }

    if variants:
        out["variants"] = variants
    if sweep_report:
        out["sweep"] = sweep_report

    if not args.no_cpu_baseline:
        from oracle import isopo_oracle as orc
        from threadpoolctl import threadpool_info
        # one projection of the block, all sequences: the one whose estimated oracle time (two fp64
        # contractions at a few hundred GFLOP/s) is nearest 12 s
        est = lambda p: 4.0 * n_tokens * p.d_in * p.d_out / 2.5e11
        sample = min(blocks[0], key=lambda p: abs(est(p) - 12.0) if est(p) <= 25.0 else 1e9 + est(p))
        Xh, Dh = wl.to_oracle(sample.X), wl.to_oracle(sample.Delta)
        t0 = time.perf_counter()
        orc.layer_step(Xh, Dh, sample.seq_offsets, sample.A, args.variant, args.lam, orc.REG_REL_TRACE,
                       chunk_rows=512)
        t_cpu = time.perf_counter() - t0
        share = total_flops / sum(algorithmic_flops(n_tokens, sample.d_in, sample.d_out, n_seq).values())
        threads = max([ti.get("num_threads", 1) for ti in threadpool_info() if ti.get("user_api") == "blas"] or [1])
        out["cpu_baseline"] = {
            "value": n_tokens / (t_cpu * share), "unit": "tokens/s", "cores": int(threads), "kind": "oracle, one projection, scaled by flops",
            "sample": f"the block's {sample.name.split('/')[-1]} projection ({sample.d_in}x{sample.d_out}, all {n_seq} sequences, "
                      f"{n_tokens} tokens) took {t_cpu:.1f} s; scaled to the whole step by the "
                      f"algorithmic-FLOP ratio {share:.1f}"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
