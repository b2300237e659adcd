#!/usr/bin/env python3
"""Benchmark of the fused Adamas decode step on one MI355X.

A "step" is one call of adamas_decode_step for one attention layer: query encode, (optional)
append, Manhattan-distance scan over the whole code plane, top-k, gather and sparse attention
(all of Algorithm 1).  Steps rotate over `--layers` distinct layer caches so that the
256 MB last-level cache cannot stand in for HBM, and are replayed from a HIP graph that holds
one sweep over all layers (launch latency of the Python caller is not what is measured).

Whole sweeps are timed, at least 200 of them whatever --steps asks for, with an event after
every replay; `value` is the median microseconds per layer.  Prints ONE JSON line with the
step's figures, the scan kernel's roofline and the CPU oracle's time on the same workload.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak
MIN_SWEEPS = 200         # timed graph replays of the fused step (each one sweep over all layers)
MIN_REPLAYS = 20         # timed graph replays of every secondary leg (scan, stream read, dense, ...)

WORKLOADS = {
    # name: (B, Hq, Hkv, context, default k, append, ragged)
    "cfg0": dict(B=1, Hq=1, Hkv=1, L=1024, k=64, append=False, ragged=False,
                 text="config 0: tiny single-head decode, batch 1, 1 query = 1 KV head, "
                      "head_dim 128, context 1024 (latency only: two launches, no bandwidth figure)"),
    "cfg1": dict(B=1, Hq=32, Hkv=32, L=32768, k=256, append=False, ragged=False,
                 text="config 1: Llama-style MHA layer decode, batch 1, 32 query = 32 KV heads, "
                      "head_dim 128, context 32768, all keys pre-encoded, no append"),
    "cfg2": dict(B=1, Hq=32, Hkv=8, L=32768, k=128, append=False, ragged=False,
                 text="config 2: GQA layer decode, batch 1, 32 query / 8 KV heads, context 32768"),
    "cfg3": dict(B=1, Hq=32, Hkv=8, L=131072, k=1024, append=True, ragged=False,
                 text="config 3: long-context decode, 32 query / 8 KV heads, context 131072 "
                      "after appending one token per step"),
    "cfg4": dict(B=16, Hq=32, Hkv=8, L=32768, k=128, append=False, ragged=True,
                 text="config 4: batched decode, 16 sequences with lengths uniform in "
                      "[8192, 32768], 32 query / 8 KV heads, ragged pool"),
    # two shapes none of the plan's thresholds were fitted on (a check of the launch plan, not a
    # configuration of the benchmark)
    "x1": dict(B=4, Hq=32, Hkv=4, L=65536, k=256, append=True, ragged=False,
               text="off-config check 1: batch 4, 32 query / 4 KV heads (group 8), context 65536, "
                    "one token appended per step"),
    "x2": dict(B=64, Hq=32, Hkv=8, L=2048, k=128, append=False, ragged=False,
               text="off-config check 2: batch 64 short sequences of 2048 tokens, 32 query / 8 KV heads"),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6400)
    ap.add_argument("--warmup", type=int, default=640)
    ap.add_argument("--config", default="cfg1", choices=sorted(WORKLOADS))
    ap.add_argument("--k", type=int, default=0, help="token budget (0: the workload's default)")
    ap.add_argument("--layers", type=int, default=32, help="distinct layer caches to rotate over")
    ap.add_argument("--variant", default="adamas",
                    choices=["adamas", "no_hadamard", "l2", "no_hadamard_l2"],
                    help="ablation switches of Section 4.4 (default: the method itself)")
    ap.add_argument("--code-bits", type=int, default=2, choices=[1, 2, 3],
                    help="bucketization granularity (Section 4.4 ablation; 2 is the method)")
    ap.add_argument("--head-dim", type=int, default=128, choices=[64, 96, 128, 160, 192, 256],
                    help="head dimension (128: the paper's models; the others run the same workload "
                         "shape with rows of that size)")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_TOKENS",
                    help="lay the cache out on randomly placed pages of this many tokens and time "
                         "adamas_decode_step_paged (0: contiguous sequences)")
    ap.add_argument("--min-sweeps", type=int, default=MIN_SWEEPS,
                    help="fewest timed graph replays of the fused step (a profiler run may want fewer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of a graph")
    ap.add_argument("--scan-only", action="store_true",
                    help="time only the scan stage (profiling aid; no JSON-contract value)")
    ap.add_argument("--encode-only", action="store_true",
                    help="profiling aid: time only the bulk key encode (adamas_encode_keys over the "
                         "rotating layers) and print its figures instead of the JSON-contract line")
    ap.add_argument("--phase-trace", action="store_true",
                    help="profiling aid: load the stamping build (python -m "
                         "paper_2510_18413_amd.build --phase-trace) and print where the time goes "
                         "inside the two kernels of the step instead of the JSON-contract line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 8 plain 256 MiB copy-like kernels (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes(B, Hq, Hkv, lens, k, append, row_bytes=32, head_dim=128):
    """Bytes the method itself must move per step: every code row once per KV head, every
    selected K and V row once per query head, q in, out back, plus the appended rows."""
    kv_row = 4 * head_dim            # one K row and one V row, bf16
    codes = Hkv * sum(lens) * row_bytes
    gather = Hq * sum(min(k, L) for L in lens) * kv_row
    small = B * Hq * (2 * head_dim + 4 * head_dim)      # q in (bf16), out back (fp32)
    app = B * Hkv * (2 * kv_row + row_bytes) if append else 0
    return codes + gather + small + app, codes


SCAN_PHASES = ["start", "length known", "query planes ready", "rows consumed",
               "distances stored", "histogram flushed (end)"]
SELECT_PHASES = ["start", "distances + histograms + length loaded", "threshold T known",
                 "first pass: candidate masks and counts", "first pass: prefix over the workgroup",
                 "compaction done", "first K/V rows arrived", "rows consumed",
                 "row groups combined", "partial stored + acknowledged", "arrival counted",
                 "merged (last workgroup only)", "end"]


def phase_trace(A, torch, np, make_graph, n_layers, args, sweeps=40):
    """Replays the graph of one sweep `sweeps` times; after each replay the trace buffers hold
    the stamps of the sweep's last layer (back-to-back kernels, as in the timed run).  Prints a
    table per kernel: when, relative to the kernel's first workgroup start, the median / 90th
    percentile / last workgroup passes each phase boundary (us, 100 MHz clock: 0.01 us steps)."""
    n_rec = 1 << 16
    dev = torch.device("cuda:0")
    tr_scan = torch.zeros(n_rec, A.TRACE_SLOTS, dtype=torch.int64, device=dev)
    tr_sel = torch.zeros(n_rec, A.TRACE_SLOTS, dtype=torch.int64, device=dev)
    A.adamas_phase_trace(tr_scan, tr_sel)
    g = make_graph(None)
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    rows = {"scan": [], "select": [], "gap": [], "scan_len": [], "select_len": []}
    for _ in range(sweeps):
        tr_scan.zero_()
        tr_sel.zero_()
        g.replay()
        torch.cuda.synchronize()
        sc, se = tr_scan.cpu().numpy(), tr_sel.cpu().numpy()
        sc, se = sc[sc[:, 0] > 0], se[se[:, 0] > 0]
        s0, e0 = sc[:, 0].min(), se[:, 0].min()
        rows["scan"].append(np.where(sc > 0, (sc - s0) * 0.01, np.nan))
        rows["select"].append(np.where(se > 0, (se - e0) * 0.01, np.nan))
        rows["gap"].append((e0 - sc.max()) * 0.01)
        rows["scan_len"].append((sc.max() - s0) * 0.01)
        rows["select_len"].append((se.max() - e0) * 0.01)
    A.adamas_phase_trace(None, None)
    out = {"config": args.config, "k": args.k, "sweeps": sweeps, "layers": n_layers,
           "scan_first_start_to_last_end_us": round(float(np.median(rows["scan_len"])), 2),
           "select_first_start_to_last_end_us": round(float(np.median(rows["select_len"])), 2),
           "scan_end_to_select_start_us": round(float(np.median(rows["gap"])), 2)}
    for name, phases in (("scan", SCAN_PHASES), ("select", SELECT_PHASES)):
        allr = np.concatenate(rows[name], axis=0)
        print("\n%s kernel: %d workgroup records per launch, %d launches; us after the kernel's "
              "first workgroup start" % (name, allr.shape[0] // sweeps, sweeps))
        print("| phase boundary | workgroups passing | median | p90 | last |")
        print("|---|---|---|---|---|")
        tab = []
        for i, ph in enumerate(phases):
            col = allr[:, i]
            col = col[~np.isnan(col)]
            if col.size == 0:
                continue
            # "last": median over launches of the latest workgroup of each launch
            last = np.median([np.nanmax(r[:, i]) for r in rows[name] if not np.all(np.isnan(r[:, i]))])
            tab.append((ph, int(col.size // sweeps), float(np.median(col)),
                        float(np.percentile(col, 90)), float(last)))
            print("| %s | %d | %.2f | %.2f | %.2f |" % tab[-1])
        out[name] = [dict(phase=t[0], workgroups=t[1], median_us=round(t[2], 2),
                          p90_us=round(t[3], 2), last_us=round(t[4], 2)) for t in tab]
    print("\nscan first start -> last end %.2f us; scan last end -> select first start %.2f us; "
          "select first start -> last end %.2f us (medians over %d launches)" % (
              out["scan_first_start_to_last_end_us"], out["scan_end_to_select_start_us"],
              out["select_first_start_to_last_end_us"], sweeps))
    print(json.dumps(out), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build measures one GPU only (every stage of the path "
                         "runs on one MI355X and no collective exists); --gpus %d is not "
                         "supported.\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    if args.phase_trace:
        trace_lib = os.path.join(ROOT, "paper_2510_18413_amd", "libadamas_trace.so")
        if not os.path.exists(trace_lib):
            raise SystemExit("build the stamping library first: python -m paper_2510_18413_amd.build "
                             "--phase-trace")
        os.environ["ADAMAS_LIBRARY"] = trace_lib
    import paper_2510_18413_amd as A
    import synth_inputs as synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    wl = WORKLOADS[args.config]
    B, Hq, Hkv, G = wl["B"], wl["Hq"], wl["Hkv"], wl["Hq"] // wl["Hkv"]
    k = args.k or wl["k"]
    append = wl["append"]
    n_layers = max(1, args.layers)
    cfg_id = int(args.config[3:]) if args.config.startswith("cfg") else 10 + int(args.config[1:])

    # ------------------------------------------------------------------ inputs
    if wl["ragged"]:
        lens = np.random.default_rng(synth.config_seed(cfg_id) + 500).integers(
            8192, wl["L"] + 1, size=B).astype(np.int32)
    else:
        lens = np.full(B, wl["L"], dtype=np.int32)
    starts = np.zeros(B, dtype=np.int64)
    pos = 0
    for b in range(B):
        starts[b] = pos
        pos += int(lens[b]) + synth.SEQ_GAP_ROWS
    pool = pos - synth.SEQ_GAP_ROWS
    max_len = int(lens.max())
    page = args.paged
    if page:
        # every sequence gets its own pages, placed by a seeded permutation; src_row maps a pool
        # row of the paged layout to the row of the contiguous layout it is filled from
        need = [(int(L) + page - 1) // page for L in lens]
        n_pages = sum(need)
        order = np.random.default_rng(synth.config_seed(cfg_id) + 900).permutation(n_pages)
        table_np = np.full((B, max(need)), -1, dtype=np.int32)
        src_row = np.zeros(n_pages * page, dtype=np.int64)
        at = 0
        for b in range(B):
            for pg in range(need[b]):
                phys = int(order[at]); at += 1
                table_np[b, pg] = phys
                tok = np.minimum(pg * page + np.arange(page), int(lens[b]) - 1)
                src_row[phys * page:(phys + 1) * page] = starts[b] + tok
        contiguous_pool, pool = pool, n_pages * page
        page_table = torch.from_numpy(table_np).to(dev)
        src_row_dev = torch.from_numpy(src_row).to(dev)
    no_hadamard = args.variant in ("no_hadamard", "no_hadamard_l2")
    squared = args.variant in ("l2", "no_hadamard_l2")
    bits = args.code_bits
    thr = {1: (0.0,), 2: synth.DEFAULT_THRESHOLDS, 3: (-1.5, -1.0, -0.5, 0.0, 0.5, 1.0, 1.5)}[bits]
    if bits != 2 and (page or squared):
        raise SystemExit("--code-bits 1/3 is benchmarked on the contiguous layout with Eq. 6 only")
    HD = args.head_dim
    cfg = A.Config.make(Hq, Hkv, pool, thr_k=thr,
                        variant=(A.VARIANT_NO_HADAMARD if no_hadamard else 0)
                        | (A.VARIANT_L2 if squared else 0), code_bits=0 if bits == 2 else bits,
                        head_dim=HD)
    row_bytes = cfg.code_row_bytes
    seq_start = torch.from_numpy(starts).to(dev)
    seq_len = torch.from_numpy(lens).to(dev)

    globals_pool = pool

    def gen_layer(layer):
        """Same recipe as synth_inputs (N(0,1) bf16, 4 outlier channels x8 per KV head, one
        needle per query head, tiny magnitudes flushed to 0), drawn on the GPU."""
        g = torch.Generator(device=dev)
        g.manual_seed(synth.config_seed(cfg_id, layer))

        def rows(n, scale):
            x = torch.randn(n, HD, generator=g, device=dev) * scale
            return torch.where(x.abs() < synth.FLUSH_BELOW, torch.zeros_like(x), x)

        pool = contiguous_pool if page else globals_pool
        K = torch.empty(Hkv, pool, HD, dtype=torch.bfloat16, device=dev)
        V = torch.empty(Hkv, pool, HD, dtype=torch.bfloat16, device=dev)
        q = torch.empty(B, Hq, HD, dtype=torch.bfloat16, device=dev)
        k_new = torch.empty(B, Hkv, HD, dtype=torch.bfloat16, device=dev) if append else None
        v_new = torch.empty(B, Hkv, HD, dtype=torch.bfloat16, device=dev) if append else None
        for h in range(Hkv):
            sk = torch.ones(HD, device=dev)
            sk[torch.randperm(HD, generator=g, device=dev)[:4]] = synth.OUTLIER_SCALE
            sv = torch.ones(HD, device=dev)
            sv[torch.randperm(HD, generator=g, device=dev)[:4]] = synth.OUTLIER_SCALE
            K[h] = rows(pool, sk).to(torch.bfloat16)
            V[h] = rows(pool, sv).to(torch.bfloat16)
            for b in range(B):
                cached = int(lens[b]) - (1 if append else 0)
                if append:
                    k_new[b, h] = rows(1, sk)[0].to(torch.bfloat16)
                    v_new[b, h] = rows(1, sv)[0].to(torch.bfloat16)
                where = torch.randperm(cached, generator=g, device=dev)[:G].tolist()
                for gq in range(G):
                    u = rows(1, sk)[0]
                    q[b, h * G + gq] = (u + synth.NEEDLE_SIGMA * torch.randn(
                        HD, generator=g, device=dev)).to(torch.bfloat16)
                    K[h, int(starts[b]) + where[gq]] = (u + synth.NEEDLE_SIGMA * torch.randn(
                        HD, generator=g, device=dev)).to(torch.bfloat16)
        return dict(q=q, K=K, V=V, k_new=k_new, v_new=v_new)

    def upload_case(case):
        def d(a):
            return None if a is None else torch.from_numpy(
                np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(dev)
        return dict(q=d(case.q), K=d(case.K), V=d(case.V), k_new=d(case.k_new), v_new=d(case.v_new))

    t_gen = time.time()
    layers = []
    case0 = None
    for layer in range(n_layers):
        if layer == 0 and args.config == "cfg1" and HD == 128:
            case0 = synth.mha_32k(layer=0)      # the numpy recipe: checked against the oracle below
            data = upload_case(case0)
        else:
            data = gen_layer(layer)
        if page:    # pure re-layout of the rows just generated
            data["K"] = data["K"].index_select(1, src_row_dev).contiguous()
            data["V"] = data["V"].index_select(1, src_row_dev).contiguous()
        data["codes"] = torch.empty(Hkv, pool, row_bytes, dtype=torch.uint8, device=dev)
        data["out"] = torch.zeros(B, Hq, HD, device=dev)
        A.adamas_encode_keys(cfg, data["K"], data["codes"], 0, pool)
        layers.append(data)
    # bulk key encode (prefill-side, not part of the timed step): median over 12 timed blocks of
    # 40 runs each over the rotating layers, after 60 untimed runs (the clocks have dropped during
    # the set-up above, and a block of a few runs is too short to time)
    def encode_block(n):
        for i in range(n):
            A.adamas_encode_keys(cfg, layers[i % n_layers]["K"], layers[i % n_layers]["codes"], 0, pool)
    encode_block(60)
    torch.cuda.synchronize()
    encode_blocks = []
    for _ in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        encode_block(40)
        e1.record()
        torch.cuda.synchronize()
        encode_blocks.append(e0.elapsed_time(e1) * 1e3 / 40)
    encode_us = sorted(encode_blocks)[len(encode_blocks) // 2]
    encode_bytes = Hkv * pool * (2 * HD + row_bytes)
    if args.encode_only:
        print(json.dumps({"bulk_encode_us": round(encode_us, 2),
                          "blocks_min_max_us": [round(min(encode_blocks), 2), round(max(encode_blocks), 2)], "rows": Hkv * pool, "bytes": encode_bytes,
                          "GBps": round(encode_bytes / encode_us / 1e3, 1),
                          "hbm_frac": round(encode_bytes / encode_us / 1e3 / HBM_PEAK_GBPS, 4),
                          "config": args.config, "head_dim": HD, "code_bits": bits}))
        return
    idx0 = torch.empty(B, Hq, k, dtype=torch.int32, device=dev)
    ws = torch.empty(A.adamas_workspace_bytes(cfg, B, max_len, k), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    def step(i, stages=None):
        d = layers[i % n_layers]
        if page:
            A.adamas_decode_step_paged(cfg, d["q"], d["K"], d["V"], d["codes"], page_table, page,
                                       seq_len, k, d["out"], max_len, ws, k_new=d["k_new"],
                                       v_new=d["v_new"],
                                       idx_out=idx0 if (i % n_layers == 0) else None,
                                       stages=A.STAGE_ALL if stages is None else stages)
            return
        A.adamas_decode_step_stages(cfg, d["q"], d["K"], d["V"], d["codes"], seq_start, seq_len, k,
                                    d["out"], max_len, ws, k_new=d["k_new"], v_new=d["v_new"],
                                    idx_out=idx0 if (i % n_layers == 0) else None, stages=stages)

    # With an append every step rewrites the same last row with the same values: the cache
    # length stays fixed, so all timed steps do identical work.

    def make_graph(stages):
        for i in range(n_layers):      # warm the code path before capture
            step(i, stages)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n_layers):
                step(i, stages)
        return g

    def sweep_plan(steps, warmup, min_sweeps):
        """Whole sweeps only: (timed sweeps, warm-up sweeps) for a request of `steps` / `warmup`
        single steps; never fewer than `min_sweeps` timed sweeps."""
        return max(min_sweeps, -(-steps // n_layers)), max(3, -(-warmup // n_layers))

    def replay_timed(g, sweeps, warm_sweeps, per_replay):
        """Replays graph `g` (per_replay launches of the thing measured) `sweeps` times with a
        HIP event after every replay, on the stream the graph runs on.  Returns the sorted
        per-launch times in us, one per replay."""
        for _ in range(warm_sweeps):
            g.replay()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(sweeps + 1)]
        ev[0].record()
        for s in range(sweeps):
            g.replay()
            ev[s + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[s].elapsed_time(ev[s + 1]) * 1e3 / per_replay for s in range(sweeps))

    def pct(sorted_us):
        n = len(sorted_us)
        return [round(sorted_us[n // 10], 3), round(sorted_us[n // 2], 3),
                round(sorted_us[(n * 9) // 10], 3)]

    def timed(stages, steps, warmup, min_sweeps=None):
        """Returns (sorted us per step of every timed sweep, steps timed).  Graph mode times whole
        sweeps over the rotating layers, whatever `steps` asks for; --eager times `steps` Python
        launches once."""
        if args.eager:
            for i in range(warmup):
                step(i, stages)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                step(i, stages)
            e1.record()
            torch.cuda.synchronize()
            return [e0.elapsed_time(e1) * 1e3 / steps], steps
        g = make_graph(stages)
        sweeps, warm = sweep_plan(steps, warmup, args.min_sweeps if min_sweeps is None else min_sweeps)
        return replay_timed(g, sweeps, warm, n_layers), sweeps * n_layers

    if args.calibrate_copy:
        # bitwise_not: one read and one write of 256 MiB, under a kernel name that is easy to
        # find in the counter output
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(7)
        dst = torch.empty_like(src)
        for _ in range(8):
            torch.bitwise_not(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.phase_trace:
        phase_trace(A, torch, np, make_graph, n_layers, args)
        return

    # ------------------------------------------------------------------ the timed region
    if args.scan_only:
        us, n = timed(A.STAGE_SCAN, args.steps, args.warmup)
        print(json.dumps({"scan_us_per_launch": round(us[len(us) // 2], 3), "timed_launches": n,
                          "config": args.config}))
        return
    step_us, timed_steps = timed(None, args.steps, args.warmup)
    us_step = step_us[len(step_us) // 2]            # median over the timed sweeps
    # dominant kernel alone (distance scan with fused query encode), same rotation
    scan_us, scan_launches = timed(A.STAGE_SCAN, args.steps // 4, args.warmup // 4, MIN_REPLAYS * 2)
    us_scan = sum(scan_us) / len(scan_us)           # average launch duration (compare rocprofv3)

    def graph_us(fn, reps=MIN_REPLAYS):
        """Sorted us per call of fn(layer_dict) over the rotating layers: one graph of a sweep,
        `reps` timed replays with a HIP event after each."""
        for d in layers:
            fn(d)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for d in layers:
                fn(d)
        return replay_timed(g, reps, 3, len(layers))

    def mean(xs):
        return sum(xs) / len(xs)

    # achievable ceiling: a read-only streaming kernel over the same code planes, same rotation
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    stream_us = mean(graph_us(lambda d: A.adamas_stream_read(d["codes"].view(-1), sink),
                              MIN_REPLAYS * 2))
    stream_gbps = Hkv * pool * row_bytes / stream_us / 1e3

    # comparison point: dense decode attention (Eq. 1 over every cached row) on the same layers
    # (contiguous layout only: the dense kernel does not read page tables)
    full_us = None
    if not page:
        full_ws = torch.empty(A.adamas_full_attn_workspace_bytes(cfg, B, max_len), dtype=torch.uint8,
                              device=dev)
        full_out = torch.zeros(B, Hq, HD, device=dev)
        full_us = mean(graph_us(lambda d: A.adamas_full_attn(
            cfg, d["q"], d["K"], d["V"], seq_start, seq_len, full_out, max_len, full_ws)))
        full_bytes = Hkv * int(lens.sum()) * 4 * HD

    # the stand-alone entry points, stage by stage (contiguous layout), next to the fused step
    stage_us = None
    if not page:
        qcodes = torch.empty(B, Hq, row_bytes, dtype=torch.uint8, device=dev)
        idx_s = torch.empty(B, Hq, k, dtype=torch.int32, device=dev)
        out_s = torch.empty(B, Hq, HD, device=dev)
        stage_us = {
            "encode_query": mean(graph_us(lambda d: A.adamas_encode_query(cfg, d["q"], qcodes))),
            "select_topk": mean(graph_us(lambda d: A.adamas_select_topk(
                cfg, qcodes, d["codes"], seq_start, seq_len, k, idx_s, max_len, ws))),
            "sparse_attn": mean(graph_us(lambda d: A.adamas_sparse_attn(
                cfg, d["q"], d["K"], d["V"], seq_start, idx_s, out_s, max_len, ws))),
        }
        stage_us = {n: round(v, 2) for n, v in stage_us.items()}
        stage_us["sum"] = round(sum(stage_us.values()), 2)

    # one layer over and over: its 32 MiB of codes and the workspace stay in the 256 MB
    # Infinity Cache, so this is NOT the HBM figure
    resident_us = mean(graph_us(lambda d: step(0)))   # n_layers launches per replay, all on layer 0

    total_bytes, code_bytes = algorithmic_bytes(B, Hq, Hkv, [int(x) for x in lens], k, append,
                                               row_bytes, HD)
    gbps_step = total_bytes / (us_step * 1e-6) / 1e9
    gbps_scan = code_bytes / (us_scan * 1e-6) / 1e9

    traffic = None
    prof = os.path.join(ROOT, "profiles", "scan_kernel_%s_pmc.md" % args.config)
    default_path = HD == 128 and bits == 2 and not page and args.variant == "adamas" and not args.k
    if default_path and os.path.exists(prof):    # the counters were read on the default path
        for line in open(prof):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    result = {
        "metric": "decode-step \u00b5s/layer at 32K ctx (encode+select+sparse attn); achieved HBM GB/s",
        "value": round(us_step, 3),
        "unit": "\u00b5s/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "timed_steps": timed_steps,
        "ms_per_step": round(us_step * 1e-3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64 transform sums and attention scores, u32 popcount distances, f32 softmax weights and accumulation, on bf16 q/K/V",
        "data": "synthetic",
        "config": {
            "workload": wl["text"].replace("head_dim 128", "head_dim %d" % HD) + ", budget k=%d, %d rotating layer caches" % (k, n_layers),
            "batch": B, "q_heads": Hq, "kv_heads": Hkv, "context": int(max_len),
            "sum_context": int(lens.sum()), "k": k, "append": append, "variant": args.variant,
            "code_bits": bits, "head_dim": HD,
            "layout": "paged, %d-token pages, random placement" % page if page else "contiguous",
            "launch": ("eager: %d launches from Python between two HIP events" % timed_steps)
            if args.eager else
            ("HIP graph of one %d-layer sweep, replayed %d times, a HIP event after every replay; "
             "value = median sweep / %d" % (n_layers, timed_steps // n_layers, n_layers)),
        },
        "achieved_hbm_GBps": round(gbps_step, 1),
        "hbm_frac_whole_step": round(gbps_step / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": total_bytes,
        "us_per_layer_p10_p50_p90": pct(step_us) if len(step_us) > 1 else None,
        "us_per_layer_mean": round(sum(step_us) / len(step_us), 3),
        "library_build_id": A.build_id(),
        "roofline": {
            "kernel": "scan_kernel (Manhattan-distance scan + fused query encode)",
            "bound": "hbm",
            "achieved": round(gbps_scan, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(gbps_scan / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "algorithmic_bytes_per_launch": code_bytes,
            "us_per_launch": round(us_scan, 3),
            "timed_launches": scan_launches,
            "us_per_launch_p10_p50_p90": pct(scan_us) if len(scan_us) > 1 else None,
            "stream_read_same_planes": {"us_per_launch": round(stream_us, 3),
                                        "GBps": round(stream_gbps, 1),
                                        "bytes_per_launch": Hkv * pool * row_bytes},
            "frac_of_stream_read": round(gbps_scan / stream_gbps, 4),
        },
    }
    result["bulk_encode"] = {"us": round(encode_us, 1), "rows": Hkv * pool,
                             "GBps": round(encode_bytes / encode_us / 1e3, 1),
                             "hbm_frac": round(encode_bytes / encode_us / 1e3 / HBM_PEAK_GBPS, 4)}
    if stage_us is not None:
        result["stages_us_standalone_entry_points"] = stage_us
    result["cache_resident_us_per_layer"] = round(resident_us, 3)
    if full_us is not None:
        result["full_attention"] = {"us_per_layer": round(full_us, 2),
                                    "GBps": round(full_bytes / full_us / 1e3, 1),
                                    "hbm_frac": round(full_bytes / full_us / 1e3 / HBM_PEAK_GBPS, 4),
                                    "speedup_of_sparse_step": round(full_us / us_step, 2)}
    # ------------------------------------------------------------------ oracle on the host
    if not args.no_cpu_baseline:
        import oracle
        hd_scope = oracle.head_dim(HD)      # the oracle computes at this head dimension below
        hd_scope.__enter__()
        if case0 is None or page:
            # pull layer 0 back to the host for the oracle
            def h(t):
                return None if t is None else t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            d0 = layers[0]
            Kh, Vh, qh = h(d0["K"]), h(d0["V"]), h(d0["q"])
            knh, vnh = h(d0["k_new"]), h(d0["v_new"])
        else:
            Kh, Vh, qh, knh, vnh = case0.K.copy(), case0.V.copy(), case0.q, None, None
        cores = oracle.max_threads()
        # sample: as many KV heads of layer 0 as keep the oracle near 10-30 s of CPU work
        n_kv = min(Hkv, max(1, int(round(Hkv * min(1.0, 2.0e6 / max(1, Hkv * int(lens.sum())))))))
        sel_kv = list(range(n_kv))
        sel_q = [hh * G + g for hh in sel_kv for g in range(G)]
        Ks, Vs = np.ascontiguousarray(Kh[sel_kv]), np.ascontiguousarray(Vh[sel_kv])
        if append:      # the device cache already holds the appended row; the oracle re-appends it
            kns, vns = np.ascontiguousarray(knh[:, sel_kv]), np.ascontiguousarray(vnh[:, sel_kv])
        else:
            kns = vns = None
        _, rows = oracle.encode_bits(Ks, thr, bits, hadamard=not no_hadamard)   # cache state, not timed
        qs = np.ascontiguousarray(qh[:, sel_q])
        # repeated for a few seconds of wall time (the step is idempotent: an append rewrites
        # the same row with the same values); the median is reported
        times, t_all = [], time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_all < 4.0 and len(times) < 50):
            t0 = time.perf_counter()
            if page:
                ref_out, ref_idx = oracle.decode_step_paged(
                    qs, Ks, Vs, rows, table_np, page, lens, k, synth.DEFAULT_THRESHOLDS,
                    synth.DEFAULT_THRESHOLDS, 1.0 / np.sqrt(float(HD)), k_new=kns, v_new=vns,
                    hadamard=not no_hadamard, squared=squared)
            elif bits != 2:
                ref_out, ref_idx, _ = oracle.decode_step_bits(
                    qs, Ks, Vs, rows, starts, lens, k, thr, thr, bits, 1.0 / np.sqrt(float(HD)),
                    k_new=kns, v_new=vns, hadamard=not no_hadamard)
            else:
                ref_out, ref_idx, _ = oracle.decode_step(
                    qs, Ks, Vs, rows, starts, lens, k, synth.DEFAULT_THRESHOLDS,
                    synth.DEFAULT_THRESHOLDS, 1.0 / np.sqrt(float(HD)), k_new=kns, v_new=vns,
                    hadamard=not no_hadamard, squared=squared)
            times.append(time.perf_counter() - t0)
        cpu_s = sorted(times)[len(times) // 2]
        oracle.set_threads(1)
        t0 = time.perf_counter()
        if bits == 2 and not page:
            oracle.decode_step(qs, Ks, Vs, rows, starts, lens, k, synth.DEFAULT_THRESHOLDS,
                               synth.DEFAULT_THRESHOLDS, 1.0 / np.sqrt(float(HD)), k_new=kns, v_new=vns,
                               hadamard=not no_hadamard, squared=squared)
            cpu_1t = time.perf_counter() - t0
        else:
            cpu_1t = None
        oracle.set_threads(cores)
        scale_up = Hkv / n_kv
        result["cpu_baseline"] = {
            "value": round(cpu_s * scale_up * 1e6, 1),
            "unit": "\u00b5s/layer",
            "cores": cores,
            "kind": "oracle",
            "single_thread_us_per_layer": None if cpu_1t is None else round(cpu_1t * scale_up * 1e6, 1),
            "cpu_model": cpu_model(),
            "sample": "one decode step of layer 0 on %d of %d KV heads (%d query heads), full "
                      "context, median of %d runs %.3f s, scaled by %.1f" % (
                          n_kv, Hkv, len(sel_q), len(times), cpu_s, scale_up),
        }
        # the same sample doubles as a full-size parity check of the timed launch configuration
        step(0)
        torch.cuda.synchronize()
        got_idx = idx0.cpu().numpy()[:, sel_q]
        got_out = layers[0]["out"].cpu().numpy()[:, sel_q]
        floor = 1e-3 * np.abs(ref_out).max(axis=-1, keepdims=True)
        rel = float(np.max(np.abs(got_out - ref_out) / np.maximum(np.abs(ref_out), floor)))
        result["parity_vs_oracle"] = {"indices_bit_exact": bool(np.array_equal(got_idx, ref_idx)),
                                      "attn_max_rel_err": rel, "heads_checked": len(sel_q)}
        hd_scope.__exit__(None, None, None)
    result["setup_seconds"] = round(t_gen, 1)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
