#!/usr/bin/env python3
"""Benchmark of the BitTrain hot path on one MI355X.

A step is one pass of the whole hot path over one batch: bt_compress (Algorithm 1),
bt_decompress (Algorithm 2) and bt_relu_backward_from_bitmap on configuration 2 of
the workload list: an fp32 convolution activation [32,256,56,56] (25.69 M elements)
with i.i.d. zero positions at 50 % sparsity (70 % and 90 % are reported in `ops`).
Inputs are resident in HBM before the timed region.  Every step works on the next of
several independent buffer sets, so that no buffer is touched again while it could
still sit in the 256 MB last-level cache ("cold"); the same-buffer ("warm") times are
reported beside them.

Prints ONE JSON line: metric/value/unit as the driver expects, plus
  roofline      HBM roofline of the dominant kernel from its algorithmic bytes
  cpu_baseline  the CPU oracle (single thread) timed on the same tensor
  ops           per-op, per-sparsity times, GB/s, roofline fractions, compression ratio
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_config2_z50.txt")


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size), or None."""
    try:
        for line in open(TRAFFIC_FILE):
            parts = line.split()
            if len(parts) >= 2 and parts[0] == kernel + "_total_bytes":
                return int(float(parts[1]))
    except OSError:
        pass
    return None



def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sets", type=int, default=8, help="independent buffer sets rotated through (cold-cache timing)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--only-z50", action="store_true", help="skip the 70 % and 90 % sparsity rows")
    ap.add_argument("--cold-only", action="store_true",
                    help="skip the same-buffer (warm) timings, so that a profiler's per-kernel average is the cold one")
    ap.add_argument("--no-step", action="store_true",
                    help="skip the combined-step loop (in it decompress reads what compress just wrote, i.e. warm data)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip configurations 1, 3, 4 and 5 and the added rows (they take about a minute; reported under "
                         "`other_configs`)")
    ap.add_argument("--all-configs", action="store_true", help="accepted for compatibility: the other configurations are on by default")
    ap.add_argument("--timeline", action="store_true",
                    help="instead of timing: one cold bt_compress and bt_decompress of configuration 2 (50 %% zeros) with the "
                         "instrumented build of the library, per-tile time stamps printed as a markdown table")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of the input tensor, as a known-size reference for counters")
    return ap.parse_args()


def timeline(bt, wl, torch, dev, sets):
    """Per-tile time stamps (the measurement-aid build of the library, libbittrain_bench.so) of one cold bt_compress
    and one cold bt_decompress of configuration 2 at 50 % zeros, as markdown on stdout."""
    import numpy as np
    from paper_2110_15362_amd import bench_aids
    bench_aids.lib()
    bt._lib, bt.LIB_PATH = None, bench_aids.LIB_PATH          # the codec calls below are the instrumented ones
    bt.lib()
    x = wl.config2(0.5)["x"].reshape(-1)
    n, K = x.numel(), max(2, sets)
    tiles = bt.bt_index_bytes(n, x.dtype) // 8
    max_passes = 256
    xs = [x.to(dev) for _ in range(K)]
    bitmaps = [torch.empty((n + 31) // 32, dtype=torch.int32, device=dev) for _ in range(K)]
    values = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(K)]
    outs = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(K)]
    nnz = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = bt.new_workspace(n, x.dtype, device=dev)
    calls = {"bt_compress": lambda i: bt.bt_compress(xs[i % K], bitmaps[i % K], values[i % K], nnz, ws),
             "bt_decompress": lambda i: bt.bt_decompress(bitmaps[i % K], values[i % K], outs[i % K], ws)}
    print("# Per-tile timeline of one cold launch: configuration 2 (fp32 [32,256,56,56]), 50 %% zeros, %d tiles\n" % tiles)
    print("Command: `python3 bench.py --timeline` (libbittrain_bench.so is built by `__graft_entry__.build()`).  One launch each,\n"
          "after a device synchronisation, so both run a few microseconds longer than the averages of the timed loops.\n")
    print("Microseconds from the first stamp of the launch, read from the 100 MHz device clock inside the kernel (the\n"
          "measurement-aid build; the stamps cost the kernel a few per cent).  `asked`: the tile's loads have been asked\n"
          "for; `counted`: its count has been published; `prefix`: the first wave of its workgroup has seen its prefix;\n"
          "`issued`: that wave has issued the tile's stores.\n")
    for name, fn in calls.items():
        for i in range(K):
            calls["bt_compress"](i)
        for i in range(3 * K):
            fn(i)
        torch.cuda.synchronize()
        buf = torch.zeros(8 * tiles + 2 * max_passes, dtype=torch.int64, device=dev)
        bench_aids.bt_timeline_set(buf, tiles, max_passes)
        fn(1)
        torch.cuda.synchronize()
        bench_aids.bt_timeline_set(None, 0, 0)
        a = buf.cpu().numpy()
        slots = tiles
        t = a[:8 * tiles].reshape(tiles, 8)
        stamped = t[:, :4][t[:, :4] != 0]
        t0 = int(stamped.min())
        us = lambda v: (np.asarray(v, dtype=np.int64) - t0) / 100.0
        print("## %s\n" % name)
        print("| tile | asked | counted | prefix | issued |\n|---|---|---|---|---|")
        for k in sorted(set(list(range(0, slots, max(1, slots // 16))) + [1022, 1023, 2046, 2047, slots - 1])):
            if k < slots:
                r = t[k]
                print("| %d | %.2f | %.2f | %.2f | %.2f |" % (k, us(r[0]), us(r[1]), us(r[2]), us(r[3])))
        print("\nLast of all tiles: asked %.2f, counted %.2f, prefix %.2f, issued %.2f.\n"
              % tuple(float(us(t[:, c].max())) for c in range(4)))
        print("| µs | tiles asked for | counted | with prefix | stores issued |\n|---|---|---|---|---|")
        end = float(us(t[:, 3].max()))
        for g in np.arange(2.0, end + 2.0, 2.0):
            print("| %.0f | %d | %d | %d | %d |" % (g, ((t[:, 0] != 0) & (us(t[:, 0]) <= g)).sum(), ((t[:, 1] != 0) & (us(t[:, 1]) <= g)).sum(),
                                                 ((t[:, 2] != 0) & (us(t[:, 2]) <= g)).sum(), ((t[:, 3] != 0) & (us(t[:, 3]) <= g)).sum()))
        p = a[8 * tiles:].reshape(max_passes, 2)
        p = p[p[:, 0] != 0]
        print("\nScanner passes that consumed counts (time, slots):", ", ".join(
            "%.2f: %d–%d" % (float(us(tm)), int(ff) >> 32, int(ff) & 0xffffffff) for tm, ff in p), "\n")
    assert torch.equal(outs[1].view(torch.int32), xs[1].view(torch.int32)), "round trip mismatch"


def other_configs(bt, wl, torch, dev, timed, args):
    """Configurations 1, 3, 4 and 5: cold per-op times and roofline fractions.  Large tensors
    get fewer buffer sets (each set of configuration 5 is 1.6 GB) but still more than the
    256 MB last-level cache between two uses of a buffer."""
    rows = []

    def one(name, x, sets, steps):
        x = x.reshape(-1)
        n, s = x.numel(), x.element_size()
        words = (n + 31) // 32
        xs = [x.to(dev) for _ in range(sets)]
        bitmaps = [torch.empty(words, dtype=torch.int32, device=dev) for _ in range(sets)]
        values = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(sets)]
        outs = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(sets)]
        nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
        ws = bt.new_workspace(n, x.dtype, device=dev)
        for k in range(sets):
            bt.bt_compress(xs[k], bitmaps[k], values[k], nnz_d, ws)
        torch.cuda.synchronize()
        nnz = int(nnz_d.item())
        alg = n * s + 4 * words + nnz * s
        tc = timed(lambda i: bt.bt_compress(xs[i % sets], bitmaps[i % sets], values[i % sets], nnz_d, ws), steps, 3)
        td = timed(lambda i: bt.bt_decompress(bitmaps[i % sets], values[i % sets], outs[i % sets], ws), steps, 3)
        tr = timed(lambda i: bt.bt_relu_backward_from_bitmap(bitmaps[i % sets], xs[i % sets], outs[i % sets]), steps, 3)
        comp = bt.bt_compressed_size(n, nnz, x.dtype)
        rows.append({"config": name, "n": n, "dtype": str(x.dtype).replace("torch.", ""), "zero_fraction": round(1 - nnz / n, 4),
                     "compression_ratio": round(n * s / comp, 4), "buffer_sets": sets,
                     "compress_us": round(tc, 2), "decompress_us": round(td, 2), "relu_backward_us": round(tr, 2),
                     "compress_roofline_frac": round(alg / tc / 1e3 / HBM_PEAK_GBPS, 4),
                     "decompress_roofline_frac": round(alg / td / 1e3 / HBM_PEAK_GBPS, 4),
                     "relu_backward_roofline_frac": round((2 * n * s + 4 * words) / tr / 1e3 / HBM_PEAK_GBPS, 4)})

    one("1: fp32 [1,64,56,56] relu(randn) (launch-latency bound)", wl.config1()["x"], 64, 200)

    # configuration 1 again, the three calls captured once in a HIP graph and replayed: what is left
    # of the launch cost when the host is out of the loop
    x = wl.config1()["x"].reshape(-1).to(dev)
    n = x.numel()
    bitmap = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev)
    values, out, gin = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = bt.new_workspace(n, x.dtype, device=dev)

    def step1():
        bt.bt_compress(x, bitmap, values, nnz_d, ws)
        bt.bt_decompress(bitmap, values, out, ws)
        bt.bt_relu_backward_from_bitmap(bitmap, x, gin)

    t_eager = timed(lambda i: step1(), 200, 10)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step1()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step1()
    t_graph = timed(lambda i: graph.replay(), 200, 10)
    assert torch.equal(out.view(torch.int32), x.view(torch.int32)), "round trip mismatch under graph replay"
    rows.append({"config": "1: the step (compress + decompress + ReLU backward) eager and as one captured HIP graph",
                 "n": n, "step_us_eager": round(t_eager, 2), "step_us_graph_replay": round(t_graph, 2)})
    del x, bitmap, values, out, gin
    one("3a: bf16 [8,2048,4096] dead feature columns", wl.config3("a")["x"], 8, 50)
    one("3b: bf16 [8,2048,4096] dead rows (whole empty tiles)", wl.config3("b")["x"], 8, 50)
    draws = None
    for p in (0.05, 0.95):
        c = wl.config5(p, draws=draws)
        draws = c["draws"]
        one("5: fp16 [256,64,112,112] zero probability %.2f" % p, c["x"], 3, 20)
    del draws
    # double precision (the format covers half, single and double): the configuration-2 tensor as fp64
    one("fp64 [32,256,56,56], 50 % zeros (configuration 2 widened to double)", wl.config2(0.5)["x"].double(), 4, 30)

    # Section 4.3 fused into Algorithm 1 (next-step row): pre-activations of configuration 2, thresholds of the paper
    pre = wl.config2(0.5)["base"].reshape(-1)
    n, sets = pre.numel(), 8
    xs = [pre.to(dev) for _ in range(sets)]
    bitmaps = [torch.empty((n + 31) // 32, dtype=torch.int32, device=dev) for _ in range(sets)]
    values = [torch.empty(n, dtype=pre.dtype, device=dev) for _ in range(sets)]
    nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = bt.new_workspace(n, pre.dtype, device=dev)
    for thr in (0.0, 0.01, 0.05, 0.1):
        bt.bt_compress_pruned(xs[0], thr, bitmaps[0], values[0], nnz_d, ws)
        torch.cuda.synchronize()
        nnz = int(nnz_d.item())
        alg = n * 4 + 4 * ((n + 31) // 32) + nnz * 4
        t = timed(lambda i: bt.bt_compress_pruned(xs[i % sets], thr, bitmaps[i % sets], values[i % sets], nnz_d, ws), 100, 5)
        rows.append({"config": "fused prune+compress of N(0,1) pre-activations [32,256,56,56] fp32, threshold %.2f" % thr,
                     "n": n, "zero_fraction": round(1 - nnz / n, 4),
                     "compression_ratio": round(n * 4 / bt.bt_compressed_size(n, nnz, pre.dtype), 4),
                     "compress_us": round(t, 2), "compress_roofline_frac": round(alg / t / 1e3 / HBM_PEAK_GBPS, 4)})
    # the activation and its stash in one pass (dense ReLU output + compressed form), against ReLU followed by compress
    outs = [torch.empty(n, dtype=pre.dtype, device=dev) for _ in range(sets)]
    t_fused = timed(lambda i: bt.bt_activation_compress(xs[i % sets], 0.0, outs[i % sets], bitmaps[i % sets], values[i % sets], nnz_d, ws), 100, 5)

    def unfused(i):
        torch.clamp_min(xs[i % sets], 0.0, out=outs[i % sets])          # ReLU into a preallocated output
        bt.bt_compress(outs[i % sets], bitmaps[i % sets], values[i % sets], nnz_d, ws)

    t_unfused = timed(unfused, 100, 5)
    bt.bt_activation_compress(xs[0], 0.0, outs[0], bitmaps[0], values[0], nnz_d, ws)
    torch.cuda.synchronize()
    nnz = int(nnz_d.item())
    alg_fused = 2 * n * 4 + 4 * ((n + 31) // 32) + nnz * 4
    rows.append({"config": "ReLU output + its compressed form in one pass (bt_activation_compress, threshold 0) on the same pre-activations",
                 "n": n, "fused_us": round(t_fused, 2), "relu_then_compress_us": round(t_unfused, 2),
                 "fused_roofline_frac": round(alg_fused / t_fused / 1e3 / HBM_PEAK_GBPS, 4)})
    del xs, bitmaps, values, outs

    # configuration 4: the 49 ResNet-50 activations, compressed in forward order and restored in
    # reverse order on one stream with one workspace; value buffers right-sized from nnz
    shapes = wl.config4_shapes()
    n_max = max(int(__import__("math").prod(sh)) for sh in shapes)
    ws = bt.new_workspace(n_max, torch.float32, device=dev)
    scratch = torch.empty(n_max, dtype=torch.float32, device=dev)
    nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
    xs, stash, dense_bytes, comp_bytes = [], [], 0, 0
    for cfg in wl.config4_tensors():
        xd = cfg["x"].reshape(-1).to(dev)
        n = xd.numel()
        bitmap = torch.empty((n + 31) // 32, dtype=torch.int32, device=dev)
        bt.bt_compress(xd, bitmap, scratch[:n], nnz_d, ws)
        nnz = int(nnz_d.item())
        xs.append(xd)
        stash.append((bitmap, torch.empty(nnz, dtype=torch.float32, device=dev), n))
        dense_bytes += 4 * n
        comp_bytes += bt.bt_compressed_size(n, nnz, torch.float32)
    outs = [torch.empty_like(xd) for xd in xs]

    def forward(i):
        for xd, (bitmap, values, n) in zip(xs, stash):
            bt.bt_compress(xd, bitmap, values, nnz_d, ws)

    def backward(i):
        for out, (bitmap, values, n) in zip(reversed(outs), reversed(stash)):
            bt.bt_decompress(bitmap, values, out, ws)

    tf = timed(forward, 5, 1)
    tb = timed(backward, 5, 1)
    # the same set, one launch for all 49 tensors (the item arrays are built once: the buffers persist)
    ns = [xd.numel() for xd in xs]
    wsb = bt.new_batch_workspace(ns, torch.float32, device=dev)
    nnz_all = torch.zeros(len(xs), dtype=torch.int64, device=dev)
    c_items = bt.compress_items(xs, [b for b, _, _ in stash], [v for _, v, _ in stash], nnz_all)
    d_items = bt.decompress_items([b for b, _, _ in stash], [v for _, v, _ in stash], outs)
    tfb = timed(lambda i: bt.bt_compress_batch(c_items, len(xs), torch.float32, wsb), 5, 1)
    tbb = timed(lambda i: bt.bt_decompress_batch(d_items, len(xs), torch.float32, wsb), 5, 1)
    assert all(torch.equal(o.view(torch.int32), xd.view(torch.int32)) for o, xd in zip(outs, xs)), "round trip mismatch"
    alg = dense_bytes + comp_bytes
    rows.append({"config": "4: ResNet-50 activation set, batch 64, fp32, 49 tensors, 70 % zeros",
                 "n": dense_bytes // 4, "dense_bytes": dense_bytes, "compressed_bytes": comp_bytes,
                 "bytes_saved": dense_bytes - comp_bytes, "saved_pct": round(100 * (1 - comp_bytes / dense_bytes), 2),
                 "compress_all_us": round(tf, 1), "decompress_all_us": round(tb, 1),
                 "compress_roofline_frac": round(alg / tf / 1e3 / HBM_PEAK_GBPS, 4),
                 "decompress_roofline_frac": round(alg / tb / 1e3 / HBM_PEAK_GBPS, 4),
                 "batched_compress_all_us": round(tfb, 1), "batched_decompress_all_us": round(tbb, 1),
                 "batched_compress_roofline_frac": round(alg / tfb / 1e3 / HBM_PEAK_GBPS, 4),
                 "batched_decompress_roofline_frac": round(alg / tbb / 1e3 / HBM_PEAK_GBPS, 4),
                 "note": "5 GB working set: every tensor is cold when its turn comes"})
    # the same set through the tile indexes: batched compression that also writes them, batched restoration from them
    indexes = [torch.empty(bt.bt_index_bytes(n, torch.float32) // 8, dtype=torch.int64, device=dev) for n in ns]
    ci_items = bt.compress_items(xs, [b for b, _, _ in stash], [v for _, v, _ in stash], nnz_all, indexes=indexes)
    di_items = bt.decompress_items([b for b, _, _ in stash], [v for _, v, _ in stash], outs, indexes=indexes)
    tci = timed(lambda i: bt.bt_compress_batch(ci_items, len(xs), torch.float32, wsb), 5, 1)
    tdi = timed(lambda i: bt.bt_decompress_batch_indexed(di_items, len(xs), torch.float32), 5, 1)
    assert all(torch.equal(o.view(torch.int32), xd.view(torch.int32)) for o, xd in zip(outs, xs)), "round trip mismatch (indexed batch)"
    # and the activation batch: prune at 0.05, dense pruned tensors written in place, compressed form beside them
    act_items = bt.compress_items(xs, [b for b, _, _ in stash], [v for _, v, _ in stash], nnz_all, dense_outs=xs)
    tact = timed(lambda i: bt.bt_compress_batch_pruned(act_items, len(xs), torch.float32, 0.05, wsb), 5, 1)
    torch.cuda.synchronize()
    kept = int(nnz_all.sum().item())
    alg_act = 2 * dense_bytes + dense_bytes // 32 + 4 * kept
    rows.append({"config": "4 again: tile indexes (batched), and the pruning batch with dense outputs (threshold 0.05, in place)",
                 "batched_compress_with_index_us": round(tci, 1), "batched_decompress_indexed_us": round(tdi, 1),
                 "batched_compress_with_index_roofline_frac": round(alg / tci / 1e3 / HBM_PEAK_GBPS, 4),
                 "batched_decompress_indexed_roofline_frac": round(alg / tdi / 1e3 / HBM_PEAK_GBPS, 4),
                 "activation_batch_us": round(tact, 1), "activation_batch_zero_fraction": round(1 - kept / (dense_bytes // 4), 4),
                 "activation_batch_roofline_frac": round(alg_act / tact / 1e3 / HBM_PEAK_GBPS, 4)})
    del xs, stash, outs, indexes

    # the codec inside a training step: 16 ReLU layers whose saved activations are 32 MiB each, with and without the stash
    import contextlib
    from paper_2110_15362_amd import autograd as ag
    layers, batch, hidden = 16, 8192, 1024
    g = torch.Generator(device=dev).manual_seed(0)
    weights = [(torch.randn(hidden, hidden, device=dev, generator=g) / hidden ** 0.5).requires_grad_() for _ in range(layers)]
    x0 = torch.randn(batch, hidden, device=dev, generator=g)

    def mlp_step(stash_on):
        ctx = ag.BitmapStash(deferred=stash_on == "deferred") if stash_on else contextlib.nullcontext()
        with ctx:
            y = x0
            for w in weights:
                y = ag.bitmap_relu(y @ w) if stash_on else torch.relu(y @ w)
            loss = y.sum()
        loss.backward()
        return ctx

    res = {}
    for stash_on in (False, True, "deferred"):
        for _ in range(3):
            ctx = mlp_step(stash_on)
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        before = torch.cuda.memory_allocated()
        t0 = time.perf_counter()
        for _ in range(10):
            ctx = mlp_step(stash_on)
        torch.cuda.synchronize()
        res[stash_on] = ((time.perf_counter() - t0) / 10 * 1e3, (torch.cuda.max_memory_allocated() - before) / 2**20,
                         ctx.stats if stash_on else None)
    rows.append({"config": "autograd stash: 16 x (matmul 8192x1024x1024 fp32 + ReLU), forward + backward, host clock",
                 "step_ms_without_stash": round(res[False][0], 2), "step_ms_with_stash": round(res[True][0], 2),
                 "step_ms_with_deferred_stash": round(res["deferred"][0], 2),
                 "peak_MiB_without_stash": round(res[False][1]), "peak_MiB_with_stash": round(res[True][1]),
                 "peak_MiB_with_deferred_stash": round(res["deferred"][1]),
                 "saved_dense_MiB": round(res[True][2]["dense_bytes"] / 2**20), "saved_stored_MiB": round(res[True][2]["stored_bytes"] / 2**20),
                 "note": "packing reads nnz and the workspace status back to right-size the value buffer: one host synchronisation per saved "
                         "tensor; the deferred stash lets them arrive behind an event and cuts the buffer to size later"})
    return rows


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (the codec has no cross-GPU step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2110_15362_amd.bittrain as bt
    from paper_2110_15362_amd import bench_aids as aids
    from paper_2110_15362_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible (there is no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    bt.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    if args.timeline:
        timeline(bt, wl, torch, dev, args.sets)
        return

    def timed(fn, iters, warm):
        """Average microseconds per call of fn(i), HIP events on the launch stream."""
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(iters):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    def timed_batches(fn, iters, warm, batches=5):
        """As timed(), with an event after every iters/batches calls: (average over all calls, median and
        minimum of the batch averages), microseconds per call.  Nothing is synchronised between batches."""
        batches = max(1, min(batches, iters))
        per = iters // batches
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(batches + 1)]
        ev[0].record(stream)
        for b in range(batches):
            for i in range(per):
                fn(b * per + i)
            ev[b + 1].record(stream)
        torch.cuda.synchronize()
        each = sorted(ev[b].elapsed_time(ev[b + 1]) * 1e3 / per for b in range(batches))
        return ev[0].elapsed_time(ev[batches]) * 1e3 / (per * batches), each[len(each) // 2], each[0]

    K = max(1, args.sets)
    levels = [0.5] if args.only_z50 else [0.5, 0.7, 0.9]
    ops, headline = [], None
    base = None
    x50_cpu = None
    for z in levels:
        cfg = wl.config2(z, base=base)
        base = cfg["base"]
        x = cfg["x"].reshape(-1)
        if z == 0.5:
            x50_cpu = x
        n, s = x.numel(), x.element_size()
        words = (n + 31) // 32
        g = torch.randn(n, generator=torch.Generator().manual_seed(12))
        xs = [x.to(dev) for _ in range(K)]
        gs = [g.to(dev) for _ in range(K)]
        bitmaps = [torch.empty(words, dtype=torch.int32, device=dev) for _ in range(K)]
        values = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(K)]     # worst-case capacity
        outs = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(K)]
        gins = [torch.empty(n, dtype=x.dtype, device=dev) for _ in range(K)]
        nnz_d = torch.zeros(1, dtype=torch.int64, device=dev)
        ws = bt.new_workspace(n, x.dtype, device=dev)
        for k in range(K):
            bt.bt_compress(xs[k], bitmaps[k], values[k], nnz_d, ws)
        torch.cuda.synchronize()
        nnz = int(nnz_d.item())
        # sanity: the round trip reproduces the input bits (full parity lives in tests/)
        bt.bt_decompress(bitmaps[0], values[0], outs[0], ws)
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int32), xs[0].view(torch.int32)), "round trip mismatch"

        alg_codec = n * s + 4 * words + nnz * s            # read n*s, write bitmap + values (and the reverse)
        alg_relu = 2 * n * s + 4 * words

        def compress(i):
            bt.bt_compress(xs[i % K], bitmaps[i % K], values[i % K], nnz_d, ws)

        def decompress(i):
            bt.bt_decompress(bitmaps[i % K], values[i % K], outs[i % K], ws)

        def relu(i):
            bt.bt_relu_backward_from_bitmap(bitmaps[i % K], gs[i % K], gins[i % K])

        def step(i):
            compress(i); decompress(i); relu(i)

        # the same pair with the tile index (8 bytes per tile written by compress, read by decompress);
        # reported beside the plain calls, not part of the step
        tiles = bt.bt_index_bytes(n, x.dtype) // 8
        indexes = [torch.empty(tiles, dtype=torch.int64, device=dev) for _ in range(K)]
        for k in range(K):
            bt.bt_compress_indexed(xs[k], bitmaps[k], values[k], nnz_d, indexes[k], ws)
        bt.bt_decompress_indexed(bitmaps[0], values[0], indexes[0], outs[0])
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int32), xs[0].view(torch.int32)), "round trip mismatch (indexed)"

        def compress_indexed(i):
            bt.bt_compress_indexed(xs[i % K], bitmaps[i % K], values[i % K], nnz_d, indexes[i % K], ws)

        def decompress_indexed(i):
            bt.bt_decompress_indexed(bitmaps[i % K], values[i % K], indexes[i % K], outs[i % K])

        row = {"sparsity": z, "n": n, "nnz": nnz, "measured_zero_fraction": round(1 - nnz / n, 5),
               "compressed_bytes": bt.bt_compressed_size(n, nnz, x.dtype), "dense_bytes": n * s,
               "compression_ratio": round(n * s / bt.bt_compressed_size(n, nnz, x.dtype), 4),
               "footprint_reduction_pct": round(100 * (1 - bt.bt_compressed_size(n, nnz, x.dtype) / (n * s)), 2)}
        timed(step, 100, 0)      # untimed: brings clocks and caches to the state the measured loops run in
        for name, fn, alg in (("compress", compress, alg_codec), ("decompress", decompress, alg_codec),
                              ("relu_backward", relu, alg_relu),
                              ("compress_indexed", compress_indexed, alg_codec + 8 * tiles),
                              ("decompress_indexed", decompress_indexed, alg_codec + 8 * tiles)):
            cold, cold_median, cold_min = timed_batches(fn, args.steps, args.warmup)
            warm = cold if args.cold_only else timed(lambda i, fn=fn: fn(0), args.steps, args.warmup)
            row[name] = {"us_cold": round(cold, 2), "us_cold_median_of_5_batches": round(cold_median, 2),
                         "us_cold_min_of_5_batches": round(cold_min, 2), "us_warm": round(warm, 2),
                         "input_GBps_cold": round(n * s / cold / 1e3, 1), "input_GBps_warm": round(n * s / warm / 1e3, 1),
                         "algorithmic_bytes": alg,
                         "roofline_frac_cold": round(alg / cold / 1e3 / HBM_PEAK_GBPS, 4),
                         "roofline_frac_warm": round(alg / warm / 1e3 / HBM_PEAK_GBPS, 4)}
        if z == 0.5:
            # what a stream with the same traffic and no dependency between workgroups gets on this GPU:
            # one tile per workgroup, 8 rows (32 KiB) read + 4 written for compress, 4 read + 8 written for
            # decompress (at 50 % zeros the compressed side is half the dense side, plus the bitmap's 3 %)
            tiles32k = n * s // 32768
            tc = timed(lambda i: aids.bt_stream_probe(xs[i % K], values[i % K], tiles32k, 8, 4), args.steps, args.warmup)
            td = timed(lambda i: aids.bt_stream_probe(values[i % K], outs[i % K], tiles32k, 4, 8), args.steps, args.warmup)
            tcp = timed(lambda i: aids.bt_stream_probe(xs[i % K], outs[i % K], tiles32k, 8, 8), args.steps, args.warmup)
            moved = tiles32k * 12 * 4096
            stream_ceiling = {"what": "dependency-free streams of the same shape (bt_stream_probe), cold",
                              "compress_like_us": round(tc, 2), "compress_like_frac": round(moved / tc / 1e3 / HBM_PEAK_GBPS, 4),
                              "decompress_like_us": round(td, 2), "decompress_like_frac": round(moved / td / 1e3 / HBM_PEAK_GBPS, 4),
                              "copy_us": round(tcp, 2), "copy_frac": round(tiles32k * 16 * 4096 / tcp / 1e3 / HBM_PEAK_GBPS, 4)}
            t_step = float("nan") if args.no_step else timed(step, args.steps, args.warmup)
            headline = {"n": n, "s": s, "nnz": nnz, "t_step_us": t_step, "row": row, "alg_codec": alg_codec,
                        "stream_ceiling": stream_ceiling}
            if args.copy_calibration:
                timed(lambda i: outs[i % K].copy_(xs[i % K]), 10, 2)
        ops.append(row)
        del xs, gs, bitmaps, values, outs, gins, indexes

    other = None
    if not args.no_other_configs:
        other = other_configs(bt, wl, torch, dev, timed, args)

    n, s, row = headline["n"], headline["s"], headline["row"]
    t_step = headline["t_step_us"]
    # dominant kernel of the step: the slower of the two codec kernels (the ReLU kernel is a plain stream)
    dom = max(("compress", "decompress"), key=lambda k: row[k]["us_cold"])
    achieved = row[dom]["algorithmic_bytes"] / row[dom]["us_cold"] / 1e3
    roofline = {"bound": "hbm", "kernel": {"compress": "compress_kernel<4, 0, false, CompressOne>", "decompress": "decompress_kernel<4, DecompressOne>"}[dom], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(dom),
                "traffic_source": (None if measured_traffic(dom) is None else
                                   "profiles/hbm_traffic_config2_z50.txt: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE of this "
                                   "kernel on this workload, each scaled by the same counter's reading for a plain copy of "
                                   "known size (a committed summary, not measured by this run)"),
                "north_star": {"target_frac": 0.70, "what": "bt_compress and bt_decompress on configuration 2 at 50 % zeros, cold",
                               "compress_frac": row["compress"]["roofline_frac_cold"],
                               "decompress_frac": row["decompress"]["roofline_frac_cold"],
                               "met": bool(min(row["compress"]["roofline_frac_cold"], row["decompress"]["roofline_frac_cold"]) >= 0.70)},
                "algorithmic_bytes_per_launch": row[dom]["algorithmic_bytes"],
                "avg_launch_us": row[dom]["us_cold"], "cache": "cold (8 rotating buffer sets)",
                "frac_warm": row[dom]["roofline_frac_warm"], "stream_ceiling": headline["stream_ceiling"]}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import cref
        xb = wl.bits(x50_cpu)
        gb = wl.bits(torch.randn(n, generator=torch.Generator().manual_seed(12)))
        t, cpu_t0 = [], time.perf_counter()
        while len(t) < 3 or (time.perf_counter() - cpu_t0 < 10.0 and len(t) < 200):     # about 10 s of CPU work
            t0 = time.perf_counter()
            o_bitmap, o_values, o_nnz = cref.compress(xb)
            cref.decompress(o_bitmap, o_values, n)
            cref.relu_backward(o_bitmap, gb)
            t.append(time.perf_counter() - t0)
        assert o_nnz == headline["nnz"]
        med = sorted(t)[len(t) // 2]
        cpu_model = None
        try:
            for line in open("/proc/cpuinfo"):
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu = {"value": round(3 * n * s / med / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle", "cpu_model": cpu_model,
               "host_cores_available": os.cpu_count(), "seconds_per_step": round(med, 3),
               "sample": "the full config-2 tensor at 50 %% sparsity (%d elements), %d repetitions (%.0f s of CPU work), median"
                         % (n, len(t), sum(t))}

    out = {
        "metric": "compress/decompress GB/s and % of HBM roofline at 50/70/90% sparsity",
        "value": round(3 * n * s / t_step / 1e3, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_step / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "config 2: fp32 activation [32,256,56,56], i.i.d. zeros, 50% sparsity, seed 1",
                   "step": "bt_compress + bt_decompress + bt_relu_backward_from_bitmap on one tensor",
                   "value_definition": "dense input bytes of the three calls (3 * n * 4) per second of step time",
                   "elements": n, "buffer_sets": K},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "ops": ops,
        "other_configs": other,
        "paper_context": "BitTrain reports footprint only (Jetson Nano, fp32): 34.20% on-board / 46.88% theoretical "
                         "reduction at 50% non-zeros, 56.27% / 71.88% at 25% non-zeros (Table 1); no throughput",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
