#!/usr/bin/env python3
"""Benchmark of the GELO obfuscated QKV projection on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that already
sits in HBM: draw a fresh mixing matrix A (Philox + Householder QR, or LU for the
non-orthogonal kinds), build the shield rows, mix U = A[H;S], project Y = U W, unmix
Z = A^-1 Y.  Prints ONE JSON line:
  value      whole-step throughput: algorithmic FLOP of the step (chain + A generation) / time
  roofline   the dominant kernel (the projection GEMM) against the MFMA peak of its dtype (against
             HBM bandwidth for decode-shaped batches of at most 128 rows), timed with events on
             the stream it runs on
  cpu_baseline  the fp64 CPU oracle timed on the host cores on a bounded sample
plus per-stage times, the chain-only rate with A already sampled, and the overhead against a
plain H W GEMM run through the same kernel.
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

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}          # MI355X dense matrix peaks
KIND_NAME = {0: "orthogonal", 1: "gaussian", 2: "conditioned", 3: "structured", 4: "block_orthogonal", 5: "reflector_product"}
BLOCK_ROWS = 256


def block_rows(n_data, k):
    """(mixed rows, data rows) of every block of the block-diagonal orthogonal kind (the library's layout restated:
    blocks of BLOCK_ROWS mixed rows; of the rows up to a cut r, floor(k r / n) are shield rows)"""
    n = n_data + k
    cuts = list(range(0, n, BLOCK_ROWS)) + [n]
    return [(r1 - r0, (r1 - k * r1 // n) - (r0 - k * r0 // n)) for r0, r1 in zip(cuts[:-1], cuts[1:])]


STRUCTURED_ROUNDS = 3


def butterfly_adds(n):
    """additions of one block Walsh-Hadamard transform of a column: m log2 m per block of the binary expansion"""
    return float(sum((1 << b) * b for b in range(n.bit_length()) if (n >> b) & 1))


def chain_flops(w):
    n, nd, d, p = w.n, w.n_data, w.d, w.p
    if w.kind == 3:      # structured A: mix and unmix are butterflies, only the projection is a product
        return 2.0 * n * d * p + STRUCTURED_ROUNDS * butterfly_adds(n) * (d + p)
    if w.kind == 4:      # block-diagonal A: mix and unmix block by block
        return 2.0 * n * d * p + sum(2.0 * r * r * d + 2.0 * dr * r * p for r, dr in block_rows(nd, w.k_shield))
    return 2.0 * n * n * d + 2.0 * n * d * p + 2.0 * nd * n * p


def gen_flops(w, attempts=1):
    n = float(w.n)
    qr = 8.0 / 3.0 * n ** 3            # Householder QR with explicit Q
    lu = 2.0 * n ** 3                  # LU + explicit inverse
    if w.kind == 4:
        return sum(8.0 / 3.0 * float(r) ** 3 for r, _ in block_rows(w.n_data, w.k_shield))
    # structured: sorting keys, no arithmetic to count; product of directly drawn reflectors: only Q is formed
    return {0: qr, 1: lu * attempts, 2: qr + lu, 3: 0.0, 5: 4.0 / 3.0 * n ** 3}[w.kind]


CAL_ELEMS = 1 << 28                                   # fp32 elements of the calibration copy: 1 GiB read, 1 GiB written
SRC_PATH = os.path.join(ROOT, "paper_2603_05035_amd", "csrc", "gemm_bf16.hip")
TRAFFIC_PATH = os.path.join(ROOT, "profiles", "gemm_project_traffic.json")


# Workloads made of several chains per step.  A step of "llama7b_bf16_layer" is one layer's two offloaded
# projections (Fig. 1: Q, K, V and O all go through the protocol): fused QKV on the hidden states, then O on
# the attention output (a second synthetic activation stands in), each with a fresh A of its own.  A step of
# "prefill_sweep_bf16" is the 32-layer prefill sweep (4096 rows per layer, even layers ORTHOGONAL + 205
# shields, odd layers CONDITIONED, fresh H, W and A per layer).  A step of "decode_sweep_bf16" is one decode
# step through 32 layers (64 tokens + 4 shields, a fresh 68 x 68 A per layer-step, 32 resident weights); the
# config's 128 steps are the default step count.
COMPOSITE = {
    "llama7b_bf16_layer": ["llama7b_bf16_prefill", "llama7b_bf16_oproj"],
    "prefill_sweep_bf16": ["sweep_bf16_orth" if l % 2 == 0 else "sweep_bf16_cond" for l in range(32)],
    "decode_sweep_bf16": ["decode_bf16"] * 32,
}


def run_composite(args, torch, np, g, wl):
    name = args.workload
    parts = [wl.WORKLOADS[x] for x in COMPOSITE[name]]
    L = len(parts)
    K = args.steps if args.steps_given else {"llama7b_bf16_layer": 48, "prefill_sweep_bf16": 2, "decode_sweep_bf16": 128}[name]
    Wm = args.warmup if args.warmup_given else {"llama7b_bf16_layer": 16, "prefill_sweep_bf16": 1, "decode_sweep_bf16": 8}[name]
    dt = torch.bfloat16
    # inputs resident in HBM: one weight per layer; hidden states per layer (the decode sweep reuses its 32
    # hidden-state buffers across steps: the chain does not look at the values)
    Hs, Ws = [], []
    for l, w in enumerate(parts):
        H32 = wl.make_hidden(w.n_data, w.d, w.seed * 1000 + l, w.outlier_channels)
        Hs.append(torch.from_numpy(H32).to(dt).cuda())
        Ws.append(torch.from_numpy(wl.make_weight(w.d, w.p, w.seed * 1000 + l)).to(dt).cuda())
    nmax = max(w.n for w in parts); pmax = max(w.p for w in parts); dmax = max(w.d for w in parts)
    U = torch.empty((nmax * dmax,), dtype=dt, device="cuda")
    Y = torch.empty((nmax * pmax,), dtype=dt, device="cuda")
    Z = torch.empty((max(w.n_data for w in parts) * pmax,), dtype=dt, device="cuda")
    def views(w):
        return (U[:w.n * w.d].view(w.n, w.d), Y[:w.n * w.p].view(w.n, w.p), Z[:w.n_data * w.p].view(w.n_data, w.p))

    depth = args.pipeline
    decode = parts[0].n <= 128
    if decode:
        # Decode step: the mixing objects of a whole step (one per layer) come from ONE launch on a side stream, a step
        # ahead of the chains that consume them; a chain is one host call (mix + project + unmix).
        depth = 2
        side = [torch.cuda.Stream() for _ in range(depth)]
        ctxs = [g.gelo_create(0, 0xBE00 + i, allow_batch_reuse=False) for i in range(depth)]
        w0 = parts[0]
        for c in ctxs:
            g.gelo_reserve(c, w0.kind, g.GELO_BF16, w0.n_data, w0.k_shield, w0.d, w0.p, 64, L)
        ring = [None] * depth

        def draw_step(step):
            slot = step % depth
            ring[slot] = g.gelo_sample_mixing_batch(ctxs[slot], w0.kind, w0.n_data, w0.k_shield, w0.d, g.GELO_BF16,
                                                    step * L, L, stream=side[slot])

        def run_step(step):
            slot = step % depth
            ms = ring[slot]
            u, y, z = views(w0)
            for l in range(L):
                g.gelo_chain(ctxs[slot], ms[l], Hs[l], Ws[l], z, u, y, w0.shield_scale)
                g.gelo_mixing_free(ctxs[slot], ms[l])
            draw_step(step + depth)

        for st_ in range(depth):
            draw_step(st_)
        step = 0
        for _ in range(Wm):
            run_step(step); step += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            run_step(step); step += 1
        torch.cuda.synchronize()
        t_step = (time.perf_counter() - t0) / K
        for slot in range(depth):
            for m in ring[slot]:
                g.gelo_mixing_free(ctxs[slot], m)
        i = (step + depth) * L
    elif all(w.kind == g.GELO_ORTHOGONAL and (w.n_data, w.k_shield, w.d) == (parts[0].n_data, parts[0].k_shield, parts[0].d)
             for w in parts):
        # every chain takes an ORTHOGONAL A of one shape: batched draws (`group` matrices per call, their factorisations
        # side by side) on side streams, `rings` groups alive - one being consumed while the others are drawn
        w0 = parts[0]
        group = next(b for b in range(min(32, K * L), 0, -1) if (K * L) % b == 0)   # divides the timed chains: exactly K L draws fall into them
        rings = 3
        depth = group * rings
        side = [torch.cuda.Stream() for _ in range(rings)]
        ctxs = [g.gelo_create(0, 0xBE00 + i, allow_batch_reuse=False) for i in range(rings)]
        for c in ctxs:                                   # sizes known ahead: nothing allocates inside the timed region
            g.gelo_reserve(c, w0.kind, g.GELO_BF16, w0.n_data, w0.k_shield, w0.d, 0, 1, group)
        ring = [None] * rings
        nxt = [0]

        def draw_group(r):
            ring[r] = g.gelo_sample_mixing_batch(ctxs[r], w0.kind, w0.n_data, w0.k_shield, w0.d, g.GELO_BF16, nxt[0], group,
                                                 stream=side[r])
            nxt[0] += group

        def chain(i):
            r, j, l = (i // group) % rings, i % group, i % L
            w = parts[l]
            if j == (Wm * L) % group:                        # the timed region opens with a draw (as in main)
                draw_group((r + rings - 1) % rings)
            m = ring[r][j]
            u, y, z = views(w)
            g.gelo_mix(ctxs[r], m, Hs[l], u, w.shield_scale)
            g.gelo_project(ctxs[r], u, Ws[l], y)
            g.gelo_unmix(ctxs[r], m, y, z)
            g.gelo_mixing_free(ctxs[r], m)
            ring[r][j] = None

        draw_group(rings - 1)                                # every context has drawn once before anything is timed
        for m in ring[rings - 1]:
            g.gelo_mixing_free(ctxs[rings - 1], m)
        ring[rings - 1] = None
        for r in range(rings - 1):
            draw_group(r)
        i = 0
        for _ in range(Wm * L):
            chain(i); i += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K * L):
            chain(i); i += 1
        torch.cuda.synchronize()
        t_step = (time.perf_counter() - t0) / K
        for r in range(rings):
            for m in (ring[r] or []):
                if m is not None:
                    g.gelo_mixing_free(ctxs[r], m)
        i = nxt[0]
    else:
        side = [torch.cuda.Stream() for _ in range(depth)]
        ctxs = [g.gelo_create(0, 0xBE00 + i, allow_batch_reuse=False) for i in range(depth)]
        for c in ctxs:                                   # sizes known ahead: nothing allocates inside the timed region
            for w in {(w.kind, w.n_data, w.k_shield, w.d): w for w in parts}.values():
                g.gelo_reserve(c, w.kind, g.GELO_BF16, w.n_data, w.k_shield, w.d, 0, 64, 1)
        ring = [None] * depth

        def draw(slot, idx):
            w = parts[idx % L]
            ring[slot] = (g.gelo_sample_mixing(ctxs[slot], w.kind, w.n_data, w.k_shield, w.d, g.GELO_BF16, w.cond_max, 64,
                                               idx, stream=side[slot]), idx)

        def chain(i):
            slot = i % depth
            m, idx = ring[slot]
            l = idx % L
            w = parts[l]
            u, y, z = views(w)
            g.gelo_mix(ctxs[slot], m, Hs[l], u, w.shield_scale)
            g.gelo_project(ctxs[slot], u, Ws[l], y)
            g.gelo_unmix(ctxs[slot], m, y, z)
            g.gelo_mixing_free(ctxs[slot], m)
            draw(slot, idx + depth)

        for slot in range(depth):
            draw(slot, slot)
        i = 0
        for _ in range(Wm * L):
            chain(i); i += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K * L):
            chain(i); i += 1
        torch.cuda.synchronize()
        t_step = (time.perf_counter() - t0) / K
        for slot in range(depth):
            g.gelo_mixing_free(ctxs[slot], ring[slot][0])

    # serial: the same chains through gelo_qkv_forward on one stream, nothing overlapped
    ctx = ctxs[0]
    base = (i + depth + 1 + L) // L * L
    Ks = max(1, min(K, 8))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(Ks * L):
        w = parts[j % L]
        u, y, z = views(w)
        g.gelo_qkv_forward(ctx, w.kind, Hs[j % L], Ws[j % L], z, k_shield=w.k_shield, shield_scale=w.shield_scale,
                           cond_max=w.cond_max, batch_id=base + j, U=u, Y=y)
    torch.cuda.synchronize()
    t_serial = (time.perf_counter() - t0) / Ks

    # the plain projections of one step through the same kernel, and per-layer stage times of the first layers
    def ev():
        return torch.cuda.Event(enable_timing=True)
    for l in range(L):
        g.gelo_project(ctx, Hs[l], Ws[l], views(parts[l])[2])
    torch.cuda.synchronize()
    a, b = ev(), ev()
    a.record()
    for _ in range(3):
        for l in range(L):
            g.gelo_project(ctx, Hs[l], Ws[l], views(parts[l])[2])
    b.record()
    torch.cuda.synchronize()
    t_plain = a.elapsed_time(b) / 3 * 1e-3
    stages = []
    bid = base + Ks * L + L
    for l in range(min(L, 2)):
        w = parts[l]
        u, y, z = views(w)
        acc = {"sample": 0.0, "mix": 0.0, "project": 0.0, "unmix": 0.0}
        reps = 5
        for r in range(reps):
            e = [ev() for _ in range(5)]
            e[0].record()
            m = g.gelo_sample_mixing(ctx, w.kind, w.n_data, w.k_shield, w.d, g.GELO_BF16, w.cond_max, 64, bid); bid += 1
            e[1].record(); g.gelo_mix(ctx, m, Hs[l], u, w.shield_scale)
            e[2].record(); g.gelo_project(ctx, u, Ws[l], y)
            e[3].record(); g.gelo_unmix(ctx, m, y, z)
            e[4].record(); torch.cuda.synchronize()
            g.gelo_mixing_free(ctx, m)
            for q, key in enumerate(("sample", "mix", "project", "unmix")):
                acc[key] += e[q].elapsed_time(e[q + 1]) / reps
        stages.append({"layer": l, "workload": w.name, **{k2: round(v, 4) for k2, v in acc.items()}})
    # the projection of layer 0 alone, for the roofline of the dominant kernel
    w0 = parts[0]
    u0, y0, _ = views(w0)
    for _ in range(20):
        g.gelo_project(ctx, u0, Ws[0], y0)
    torch.cuda.synchronize()
    pairs = []
    for _ in range(50):
        a, b = ev(), ev(); a.record(); g.gelo_project(ctx, u0, Ws[0], y0); b.record(); pairs.append((a, b))
    torch.cuda.synchronize()
    t_proj = sum(x.elapsed_time(y_) for x, y_ in pairs) / len(pairs) * 1e-3
    for c in ctxs:
        g.gelo_destroy(c)

    f_chain = sum(chain_flops(w) for w in parts)
    f_gen = sum(gen_flops(w) for w in parts)
    f_plain = sum(2.0 * w.n_data * w.d * w.p for w in parts)
    peak = PEAK_TFLOPS["bf16"]
    result = {
        "metric": "GELO QKV-forward TFLOP/s (whole step: A generation + shields + mix + project + unmix)",
        "value": (f_chain + f_gen) / t_step / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "chains_per_step": L, "parts": sorted({w.name for w in parts}),
                   "step": {"llama7b_bf16_layer": "one layer: fused QKV projection, then O projection, a fresh A each",
                            "prefill_sweep_bf16": "one 32-layer prefill sweep (4096 rows per layer; even layers orthogonal + 205 shields, odd layers conditioned)",
                            "decode_sweep_bf16": "one decode step through 32 layers (64 tokens + 4 shields, fresh 68 x 68 A per layer-step)"}[name]},
        "pipeline": {"depth": depth, "serial_ms_per_step": t_serial * 1e3, "serial_steps_timed": Ks,
                     "note": "A for the next chains is drawn on side streams while the chains run; every timed chain draws one A and consumes one"},
        "us_per_chain": t_step / L * 1e6, "serial_us_per_chain": t_serial / L * 1e6,
        "frac_of_mfma_peak_whole_step": (f_chain + f_gen) / t_step / 1e12 / peak,
        "plain_ms_per_step": t_plain * 1e3,
        "overhead_vs_plain_gemm_pct": {"whole_step": (t_step / t_plain - 1.0) * 100.0, "whole_step_serial": (t_serial / t_plain - 1.0) * 100.0,
                                       "flop_ratio_floor": (f_chain / f_plain - 1.0) * 100.0},
        "useful_tflops": f_plain / t_step / 1e12,
        "stage_ms_first_layers": stages,
    }
    if decode:
        b_proj = 2.0 * (w0.n * w0.d + w0.d * w0.p + w0.n * w0.p)
        result["roofline"] = {"kernel": "gemm (project Y = U W), skinny path", "bound": "hbm", "achieved": b_proj / t_proj / 1e9,
                              "peak": 8000.0, "unit": "GB/s", "frac": b_proj / t_proj / 1e9 / 8000.0, "traffic": None,
                              "avg_launch_us": t_proj * 1e6}
        result["w_stream_floor_us_per_chain"] = 2.0 * w0.d * w0.p / 8e12 * 1e6
        # HBM rate of the two small-n mixing calls (algorithmic bytes of eq. 1 / eq. 3: operands read once, result written once)
        st0 = stages[0]
        b_mix = 2.0 * (w0.n * w0.n + w0.n_data * w0.d + w0.k_shield * w0.d + w0.n * w0.d)
        b_unmix = 2.0 * (w0.n_data * w0.n + w0.n * w0.p + w0.n_data * w0.p)
        result["small_n_mixing"] = {"sample_us": st0["sample"] * 1e3, "mix_us": st0["mix"] * 1e3, "unmix_us": st0["unmix"] * 1e3,
                                    "mix_GBps": b_mix / (st0["mix"] * 1e-3) / 1e9, "unmix_GBps": b_unmix / (st0["unmix"] * 1e-3) / 1e9,
                                    "peak_GBps": 8000.0,
                                    "note": "one draw alone costs sample_us; a decode step draws its 32 in one launch, a step ahead"}
    else:
        f_proj = 2.0 * w0.n * w0.d * w0.p
        result["roofline"] = {"kernel": "gemm (project Y = U W) of the step's first chain", "bound": "mfma", "achieved": f_proj / t_proj / 1e12,
                              "peak": peak, "unit": "TFLOP/s", "frac": f_proj / t_proj / 1e12 / peak, "traffic": None,
                              "avg_launch_us": t_proj * 1e6}
    if not args.no_cpu_baseline:
        from oracle import gelo_oracle as oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([t.get("num_threads", 1) for t in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        # bounded sample: the first chain of the step on at most 1024 of its rows
        rows = min(w0.n_data, 1024)
        ks = w0.k_shield if rows == w0.n_data else int(round(0.05 * rows)) if w0.k_shield > 0 else 0
        H64, W64 = Hs[0][:rows].double().cpu().numpy(), Ws[0].double().cpu().numpy()
        t0 = time.perf_counter()
        ref = oracle.qkv_forward(w0.kind, w0.seed, 0, H64, W64, k_shield=ks, shield_scale=w0.shield_scale, cond_max=w0.cond_max)
        t_cpu = time.perf_counter() - t0
        ns = rows + ks
        f_s = 2.0 * ns * ns * w0.d + 2.0 * ns * w0.d * w0.p + 2.0 * rows * ns * w0.p + 8.0 / 3.0 * float(ns) ** 3
        result["cpu_baseline"] = {"value": f_s / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle", "seconds": t_cpu,
                                  "sample": f"one fp64 oracle chain (sampling + QR + shields + mix + project + unmix) of the step's first "
                                            f"projection on {rows} data rows + {ks} shield rows (d={w0.d}, p={w0.p})",
                                  "check_rel_err_vs_plain": float(np.linalg.norm(ref["Z"] - H64 @ W64) / np.linalg.norm(H64 @ W64))}
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="llama7b_bf16_prefill")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--draw-batch", type=int, default=32, help="ORTHOGONAL: mixing matrices per batched draw (its factorisations run side by side)")
    ap.add_argument("--pipeline", type=int, default=24, help="mixing matrices drawn ahead on side streams")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run a plain elementwise copy of known size (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    args.steps_given, args.warmup_given = args.steps is not None, args.warmup is not None
    args.steps = 64 if args.steps is None else args.steps
    args.warmup = 32 if args.warmup is None else args.warmup
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_05035_amd import binding as g
    from paper_2603_05035_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    # The interpreter's cyclic garbage collector stays off while the bench runs: a full collection over the
    # modules loaded above takes about 40 ms of host time, fell into the timed loop of the decode sweep
    # (a one-off stall worth 12 us per layer-step over 128 steps) and measures nothing of the library.
    import gc
    gc.collect()
    gc.disable()
    if args.workload in COMPOSITE:
        return run_composite(args, torch, np, g, wl)
    w = wl.WORKLOADS[args.workload]
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    H32, W32 = wl.make_inputs(w)
    H = torch.from_numpy(H32).to(tdt).cuda()
    W = torch.from_numpy(W32).to(tdt).cuda()
    n, nd, d, p, k = w.n, w.n_data, w.d, w.p, w.k_shield
    U = torch.empty((n, d), dtype=tdt, device="cuda")
    Y = torch.empty((n, p), dtype=tdt, device="cuda")
    Z = torch.empty((nd, p), dtype=tdt, device="cuda")
    Yplain = torch.empty((nd, p), dtype=tdt, device="cuda")
    code = g.GELO_BF16 if w.dtype == "bf16" else g.GELO_F32
    ctx = g.gelo_create(0, w.seed, allow_batch_reuse=False)
    K, Wm = args.steps, args.warmup
    next_batch = [0]

    def step():
        g.gelo_qkv_forward(ctx, w.kind, H, W, Z, k_shield=k, shield_scale=w.shield_scale, cond_max=w.cond_max,
                           batch_id=next_batch[0], U=U, Y=Y)
        next_batch[0] += 1

    # ---- whole step, one stream, nothing overlapped (latency of a cold batch) ----
    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    t_serial = (time.perf_counter() - t0) / K

    # ---- whole step, pipelined: A does not depend on H, so the trusted side draws the mixing matrices
    # of the next batches on side streams (one context = one workspace per stream) while the chain of
    # the current batch runs.  Every timed step still generates one fresh A and consumes one.
    main = torch.cuda.current_stream()

    def pipelined_batched(kind):
        """batched draws: `group` matrices per call (their factorisations share every launch), `rings` groups alive:
        one being consumed while the others are drawn on side streams.  A group is drawn at every step whose
        number is the warm-up count modulo the group size (so the first timed step issues one: a short timed
        region then overlaps its draws with its chains as a long one does); the group size divides K, so ANY K
        consecutive steps - the timed region - issue exactly K / group draw calls = K draws, and K chains.
        Returns (seconds per step, group, matrices alive)."""
        bid = [0]
        group = next(b for b in range(min(max(1, args.draw_batch), K), 0, -1) if K % b == 0)
        rings = 3
        side = [torch.cuda.Stream() for _ in range(rings)]
        ctxs = [g.gelo_create(0, w.seed + 1 + i, allow_batch_reuse=False) for i in range(rings)]
        for c in ctxs:
            g.gelo_reserve(c, kind, code, nd, k, d, p, 1, group)     # nothing allocates inside the timed region
        ring = [None] * rings

        def draw_group(r):
            ring[r] = g.gelo_sample_mixing_batch(ctxs[r], kind, nd, k, d, code, bid[0], group, stream=side[r])
            bid[0] += group

        def pstep(i):
            r, j = (i // group) % rings, i % group
            if j == Wm % group:                                     # the timed region opens with a draw and overlaps it whole
                draw_group((r + rings - 1) % rings)                 # the group consumed before this one is replaced
            m = ring[r][j]
            g.gelo_mix(ctxs[r], m, H, U, w.shield_scale)             # waits for the draw through the object's event
            g.gelo_project(ctxs[r], U, W, Y)
            g.gelo_unmix(ctxs[r], m, Y, Z)
            g.gelo_mixing_free(ctxs[r], m)
            ring[r][j] = None

        # every context has drawn once before anything is timed (a context's first batched draw costs its host
        # thread several milliseconds); the last one's objects go back unused
        draw_group(rings - 1)
        for m in ring[rings - 1]:
            g.gelo_mixing_free(ctxs[rings - 1], m)
        ring[rings - 1] = None
        for r in range(rings - 1):                                  # two groups ahead; the third is drawn at step Wm % group
            draw_group(r)
        for i in range(Wm):
            pstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(Wm, Wm + K):
            pstep(i)
        torch.cuda.synchronize()              # exactly K draws and K chains were issued and have finished in the region
        t = (time.perf_counter() - t0) / K
        for r in range(rings):
            for m in (ring[r] or []):
                if m is not None:
                    g.gelo_mixing_free(ctxs[r], m)
        for c in ctxs:
            g.gelo_destroy(c)
        return t, group, group * rings

    if w.kind in (g.GELO_ORTHOGONAL, g.GELO_BLOCK_ORTHOGONAL, g.GELO_REFLECTOR_PRODUCT):
        t_step, group, depth = pipelined_batched(w.kind)
    else:
        bid = [0]
        group = 1
        depth = args.pipeline
        side = [torch.cuda.Stream() for _ in range(depth)]
        ctxs = [g.gelo_create(0, w.seed + 1 + i, allow_batch_reuse=False) for i in range(depth)]
        ring = [None] * depth

        def draw(slot):
            ring[slot] = g.gelo_sample_mixing(ctxs[slot], w.kind, nd, k, d, code, w.cond_max, 64, bid[0], stream=side[slot])
            bid[0] += 1

        def pstep(i):
            slot = i % depth
            m = ring[slot]
            g.gelo_mix(ctxs[slot], m, H, U, w.shield_scale)          # waits for the draw through the object's event
            g.gelo_project(ctxs[slot], U, W, Y)
            g.gelo_unmix(ctxs[slot], m, Y, Z)
            g.gelo_mixing_free(ctxs[slot], m)
            draw(slot)                                              # refill the slot for batch i + depth

        for slot in range(depth):
            draw(slot)
        for i in range(Wm):
            pstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(Wm, Wm + K):
            pstep(i)
        torch.cuda.synchronize()              # exactly K draws and K chains were issued and have finished in the region
        t_step = (time.perf_counter() - t0) / K
        for slot in range(depth):
            g.gelo_mixing_free(ctxs[slot], ring[slot])
        for c in ctxs:
            g.gelo_destroy(c)
    # The same step with the orthogonal A drawn as a product of reflectors (the same distribution of A, no factorisation):
    # reported beside the headline figure, which keeps the QR.
    t_alt = None
    if w.kind == g.GELO_ORTHOGONAL and n > 128:
        t_alt = pipelined_batched(g.GELO_REFLECTOR_PRODUCT)[0]

    # ---- per-stage times with events on the launch stream ----
    def ev():
        return torch.cuda.Event(enable_timing=True)

    stage = {"sample": 0.0, "mix": 0.0, "project": 0.0, "unmix": 0.0, "plain": 0.0}
    attempts = []
    for i in range(K):
        e = [ev() for _ in range(7)]
        e[0].record()
        m = g.gelo_sample_mixing(ctx, w.kind, nd, k, d, code, w.cond_max, 64, next_batch[0])
        next_batch[0] += 1
        e[1].record()
        g.gelo_mix(ctx, m, H, U, w.shield_scale)
        e[2].record()
        g.gelo_project(ctx, U, W, Y)
        e[3].record()
        g.gelo_unmix(ctx, m, Y, Z)
        e[4].record()
        g.gelo_project(ctx, H, W, Yplain)
        e[5].record()
        torch.cuda.synchronize()
        if i == 0 and w.kind == 1:
            attempts.append(g.gelo_mixing_export(ctx, m, n, k, d, want_shields=False)[3] + 1)
        g.gelo_mixing_free(ctx, m)
        for name, a, b in (("sample", 0, 1), ("mix", 1, 2), ("project", 2, 3), ("unmix", 3, 4), ("plain", 4, 5)):
            stage[name] += e[a].elapsed_time(e[b]) / K
    t_chain = (stage["mix"] + stage["project"] + stage["unmix"]) * 1e-3

    # ---- the dominant kernel alone: the projection GEMM, one launch per event pair ----
    for _ in range(30):                       # long enough for the clocks to settle under this kernel's load
        g.gelo_project(ctx, U, W, Y)
    torch.cuda.synchronize()
    pairs = []
    for _ in range(max(K, 50)):
        a, b = ev(), ev()
        a.record()
        g.gelo_project(ctx, U, W, Y)
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    t_proj = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs) * 1e-3

    f_chain, f_gen = chain_flops(w), gen_flops(w, attempts[0] if attempts else 1)
    f_proj = 2.0 * n * d * p
    peak = PEAK_TFLOPS[w.dtype]
    result = {
        "metric": "GELO QKV-forward TFLOP/s (whole step: A generation + shields + mix + project + unmix)",
        "value": (f_chain + f_gen) / t_step / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": t_step * 1e3,
        "pipeline": {"depth": depth, "draws_per_call": group,
                     "note": "A for the next batches is drawn on side streams while the chain runs (ORTHOGONAL: draws_per_call "
                             "matrices per batched call, their factorisations side by side); each timed step draws one A and consumes one",
                     "serial_ms_per_step": t_serial * 1e3, "serial_tflops": (f_chain + f_gen) / t_serial / 1e12},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_data": nd, "k_shield": k, "n": n, "d": d, "p": p,
                   "mixing": KIND_NAME[w.kind], "shield_scale": w.shield_scale},
        "frac_of_mfma_peak_whole_step": (f_chain + f_gen) / t_step / 1e12 / peak,
        "chain_only": {"tflops": f_chain / t_chain / 1e12, "frac_of_mfma_peak": f_chain / t_chain / 1e12 / peak,
                       "ms": t_chain * 1e3, "note": "mix+project+unmix with A already sampled"},
        "stage_ms": {kk: round(v, 4) for kk, v in stage.items()},
        "overhead_vs_plain_gemm_pct": {"whole_step": (t_step * 1e3 / stage["plain"] - 1.0) * 100.0,
                                       "whole_step_serial": (t_serial * 1e3 / stage["plain"] - 1.0) * 100.0,
                                       "chain_only": (t_chain * 1e3 / stage["plain"] - 1.0) * 100.0,
                                       "flop_ratio_floor": (f_chain / (2.0 * nd * d * p) - 1.0) * 100.0},
        "useful_tflops": 2.0 * nd * d * p / t_step / 1e12,
        "roofline": {"kernel": "gemm (project Y = U W)", "bound": "mfma", "achieved": f_proj / t_proj / 1e12,
                     "peak": peak, "unit": "TFLOP/s", "frac": f_proj / t_proj / 1e12 / peak, "traffic": None,
                     "avg_launch_us": t_proj * 1e6},
    }

    if t_alt is not None:
        f_alt = f_chain + 4.0 / 3.0 * float(n) ** 3
        result["same_law_cheaper_draw"] = {
            "mixing": KIND_NAME[5], "ms_per_step": t_alt * 1e3, "tflops": f_alt / t_alt / 1e12,
            "overhead_vs_plain_gemm_pct": (t_alt * 1e3 / stage["plain"] - 1.0) * 100.0,
            "note": "the same pipelined step with A drawn as a product of reflectors built from the Gaussian's raw columns: Haar-distributed "
                    "like the QR factor, (4/3) n^3 operations, no chain of panels; `value` above keeps the Householder QR"}

    if w.dtype == "bf16" and n > 128:
        # the ceiling the published peak leaves out: matrix instructions from registers only, every wave of every CU
        # (no memory, no LDS, no barrier), measured here and now; the clock settles under the load, so the launches
        # are long (about 10 ms each)
        sec, flop = g.gelo_measure_matrix_rate(ctx, False, 20000, 5)
        result["roofline"]["matrix_only_ceiling"] = {"achieved": flop / sec / 1e12, "unit": "TFLOP/s", "frac_of_peak": flop / sec / 1e12 / peak,
                                                     "kernel_frac_of_ceiling": f_proj / t_proj / (flop / sec),
                                                     "note": "v_mfma_f32_32x32x16_bf16 only, 8 accumulator tiles per wave, 2 waves per SIMD, 256 CUs"}

    if w.dtype == "bf16" and d % 128 == 0 and n > 128:
        # the same projection with E4M3 operands (not part of the step above: its error is outside the bf16 contract):
        # one call = row quantisation of U + the 8-bit product; W was prepared once, outside the timed region
        Wq = g.gelo_prepare_weight_fp8(ctx, W)
        for _ in range(20):
            g.gelo_project_fp8(ctx, U, Wq, p, Y)
        torch.cuda.synchronize()
        pairs8 = []
        for _ in range(50):
            a8, b8 = ev(), ev()
            a8.record(); g.gelo_project_fp8(ctx, U, Wq, p, Y); b8.record()
            pairs8.append((a8, b8))
        torch.cuda.synchronize()
        t8 = sum(x.elapsed_time(y_) for x, y_ in pairs8) / len(pairs8) * 1e-3
        result["fp8_projection"] = {"kernel": "quantise U per row + gemm_fp8 (project Y = U W, E4M3 operands, float accumulation)",
                                    "bound": "mfma", "achieved": f_proj / t8 / 1e12, "peak": 5000.0, "unit": "TFLOP/s",
                                    "frac": f_proj / t8 / 1e12 / 5000.0, "call_us": t8 * 1e6, "bf16_call_us": t_proj * 1e6,
                                    "note": "error of Z with this projection: 4e-2 .. 7e-2 relative Frobenius (8-bit operands), outside the 2e-2 bound"}
        sec8, flop8 = g.gelo_measure_matrix_rate(ctx, True, 20000, 5)
        result["fp8_projection"]["matrix_only_ceiling"] = {"achieved": flop8 / sec8 / 1e12, "unit": "TFLOP/s", "frac_of_peak": flop8 / sec8 / 1e12 / 5000.0,
                                                           "note": "v_mfma_f32_32x32x64_f8f6f4 (E4M3) only, same shape of loop"}

    if w.kind in (0, 1, 2, 5):
        # A generation against the float matrix peak: the factorisations' trailing updates run on the float MFMA
        # path; their panels are bound by the latency of one workgroup, which is what keeps the fraction low
        t_gen = stage["sample"] * 1e-3
        result["a_gen"] = {"kernel": {0: "Philox + Householder QR with explicit Q", 1: "Philox + pivoted LU + inverse + condition estimate (per accepted draw)",
                                      2: "Householder QR + pivoted LU + inverse + condition estimate",
                                      5: "Philox + reflectors from the raw columns + their product"}[w.kind],
                           "bound": "mfma", "flop": f_gen, "ms": t_gen * 1e3, "achieved": f_gen / t_gen / 1e12, "peak": PEAK_TFLOPS["f32"],
                           "unit": "TFLOP/s", "frac": f_gen / t_gen / 1e12 / PEAK_TFLOPS["f32"],
                           "pipelined_ms_per_draw": t_step * 1e3,
                           "note": "one draw alone on one stream; pipelined_ms_per_draw bounds it from above when draws of other batches overlap"}
        if w.kind in (g.GELO_ORTHOGONAL, g.GELO_REFLECTOR_PRODUCT) and n > 128:
            # the same factorisation as throughput work: `group` draws in one batched call (side by side in the same
            # launches), nothing else on the GPU
            bctx = g.gelo_create(0, w.seed + 77, allow_batch_reuse=False)
            g.gelo_reserve(bctx, w.kind, code, nd, k, d, 0, 1, group)
            tb = []
            for rep in range(3):
                e0, e1 = ev(), ev()
                e0.record()
                ms_ = g.gelo_sample_mixing_batch(bctx, w.kind, nd, k, d, code, rep * group, group)
                e1.record()
                torch.cuda.synchronize()
                tb.append(e0.elapsed_time(e1) * 1e-3)
                for m_ in ms_:
                    g.gelo_mixing_free(bctx, m_)
            g.gelo_destroy(bctx)
            t_b = min(tb[1:]) / group
            result["a_gen"]["batched"] = {"draws_per_call": group, "ms_per_draw": t_b * 1e3, "achieved": f_gen / t_b / 1e12,
                                          "frac": f_gen / t_b / 1e12 / PEAK_TFLOPS["f32"],
                                          "note": "gelo_sample_mixing_batch alone on the GPU: the chain of panels is shared, the strips of all matrices fill the chip"}

    if n <= 128:
        # decode-shaped batches: the projection streams W once and does almost no arithmetic per byte
        # (about 2 n FLOP per byte of W), so it is bound by HBM, not by the matrix cores
        esz = 2 if w.dtype == "bf16" else 4
        b_proj = float(esz) * (n * d + d * p + n * p)
        result["roofline"] = {"kernel": "gemm (project Y = U W), skinny path", "bound": "hbm",
                              "achieved": b_proj / t_proj / 1e9, "peak": 8000.0, "unit": "GB/s",
                              "frac": b_proj / t_proj / 1e9 / 8000.0, "traffic": None, "avg_launch_us": t_proj * 1e6}

    if n <= 128:
        # HBM rate of the two small-n mixing calls of a decode-shaped batch (algorithmic bytes of eq. 1 / eq. 3:
        # every operand read once, the result written once; the stage times include the shield kernels of mix)
        esz = 2 if w.dtype == "bf16" else 4
        a_bytes = 0.0 if w.kind == 3 else float(esz) * n * n            # the structured kind reads tables, not a matrix
        b_mix = a_bytes + float(esz) * (nd * d + k * d + n * d)
        b_unmix = (a_bytes * nd / n) + float(esz) * (n * p + nd * p)
        result["small_n_mixing"] = {"mix_GBps": b_mix / (stage["mix"] * 1e-3) / 1e9, "mix_us": stage["mix"] * 1e3,
                                    "unmix_GBps": b_unmix / (stage["unmix"] * 1e-3) / 1e9, "unmix_us": stage["unmix"] * 1e3,
                                    "peak_GBps": 8000.0,
                                    "note": "both calls move about a megabyte and are bound by launch latency, not by HBM"}

    if w.kind == 3:
        # The second kernel of a structured step: the transform behind unmix (one launch, timed by the stage
        # events above).  Its butterflies are plain float additions on the vector ALUs; the peak is what
        # 256 CUs x 64 lanes x 2.4 GHz can issue when every instruction is a useful, unpacked addition.
        esz = 2 if w.dtype == "bf16" else 4
        t_un = stage["unmix"] * 1e-3
        adds = STRUCTURED_ROUNDS * butterfly_adds(n) * p
        bytes_un = float(esz) * (n * p + nd * p)
        alu_peak = 256 * 64 * 2.4e9 / 1e12
        result["transform"] = {"kernel": "structured_apply (unmix Z = A^T Y, shield rows dropped)", "bound": "alu",
                               "achieved": adds / t_un / 1e12, "peak": alu_peak, "unit": "Tadd/s",
                               "frac": adds / t_un / 1e12 / alu_peak,
                               "hbm_GBps": bytes_un / t_un / 1e9, "hbm_frac": bytes_un / t_un / 1e9 / 8000.0,
                               "launch_us": t_un * 1e6}

    # HBM traffic of the projection GEMM from the committed rocprofv3 counter runs; only valid for the
    # kernel source those runs were taken on
    try:
        import hashlib
        rec = json.load(open(TRAFFIC_PATH))
        src = open(SRC_PATH, "rb").read()
        if rec.get("workload") == w.name and rec.get("kernel_source_sha1") == hashlib.sha1(src).hexdigest():
            result["roofline"]["traffic"] = rec["traffic_bytes_per_launch"]
            result["roofline"]["traffic_source"] = ("profiles/gemm_project_traffic.json: counters taken in an earlier run on this "
                                                   "kernel source (matched by its SHA-1), not measured in this run")
    except Exception:
        pass

    if args.traffic_calibration:
        src_t = torch.ones(CAL_ELEMS, dtype=torch.float32, device="cuda")
        dst_t = torch.empty_like(src_t)
        for _ in range(3):
            torch.mul(src_t, 1.0, out=dst_t)
        torch.cuda.synchronize()
        del src_t, dst_t

    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host cores, float64: one whole step (its own Philox sampling,
        # Householder QR / LU, shields, mix, project, unmix) of this workload.  For n above 2200 the
        # Python-level QR loop alone would take minutes, so the sample is then the first 1024 data rows.
        from oracle import gelo_oracle as oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([t.get("num_threads", 1) for t in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        rows = nd if n <= 2200 else 1024
        ks = k if rows == nd else int(round(0.05 * rows)) if k > 0 else 0
        H64, W64 = H[:rows].double().cpu().numpy(), W.double().cpu().numpy()
        t0 = time.perf_counter()
        ref = oracle.qkv_forward(w.kind, w.seed, 0, H64, W64, k_shield=ks, shield_scale=w.shield_scale,
                                 cond_max=w.cond_max)
        t_cpu = time.perf_counter() - t0
        ns = rows + ks
        f_chain_s = 2.0 * ns * ns * d + 2.0 * ns * d * p + 2.0 * rows * ns * p
        if w.kind == 3:
            f_chain_s = 2.0 * ns * d * p + STRUCTURED_ROUNDS * butterfly_adds(ns) * (d + p)
        f_gen_s = {0: 8.0 / 3.0, 1: 2.0 * (ref["info"]["attempt"] + 1), 2: 8.0 / 3.0 + 2.0, 3: 0.0, 4: 0.0, 5: 4.0 / 3.0}[w.kind] * float(ns) ** 3
        if w.kind == 4:
            f_chain_s = 2.0 * ns * d * p + sum(2.0 * r * r * d + 2.0 * dr * r * p for r, dr in block_rows(rows, ks))
            f_gen_s = sum(8.0 / 3.0 * float(r) ** 3 for r, _ in block_rows(rows, ks))
        result["cpu_baseline"] = {
            "value": (f_chain_s + f_gen_s) / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": t_cpu,
            "sample": f"one whole fp64 oracle step (sampling + QR/LU + shields + mix + project + unmix) on "
                      f"{rows} data rows + {ks} shield rows (n={ns}, d={d}, p={p})"
                      + ("" if rows == nd else " - a reduced batch, the full n would take minutes in the oracle's QR loop"),
            "check_rel_err_vs_plain": float(np.linalg.norm(ref["Z"] - H64 @ W64) / np.linalg.norm(H64 @ W64))}
    g.gelo_destroy(ctx)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
